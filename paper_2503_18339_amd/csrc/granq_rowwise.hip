// Row-wise fake-quantization of many small matrices in one launch: channel-wise
// weight quantization (Sec. 5.1 of the paper) for all layers of a network at once.
// One block per row (output channel): min/max over the row (Eq. 4 with the row as
// the channel), scale and zero-point (Eq. 2), then quantize-dequantize (Eq. 1, 6).
// Rows that are a whole number of 16-byte vectors move as vectors, and a row of up to 2048
// vectors stays in the block's registers between the two steps (one read); other rows are
// read twice, the second sweep from the cache.
#include <hip/hip_runtime.h>
#include <float.h>
#include <stdint.h>

#include "granq.h"
#include "granq_device.h"
#include "granq_launch.h"
#include "granq_block.h"

namespace granq {

constexpr int kMaxItems = 32;       // descriptors per launch (passed by value)

struct RowqBatch {
    granq_rowq_item_t item[kMaxItems];
    int64_t first_row[kMaxItems + 1];   // prefix sums of rows: block b serves the item with
    int32_t count;                      // first_row[i] <= b < first_row[i + 1]
};

struct RowqBwdBatch {
    granq_rowq_bwd_item_t item[kMaxItems];
    int64_t first_row[kMaxItems + 1];
    int32_t count;
};

// Item of block b (block-uniform scan over at most 32 entries).
__device__ inline int find_item(const int64_t *first_row, int count, int64_t b) {
    int i = 0;
    while (i + 1 < count && b >= first_row[i + 1]) ++i;
    return i;
}

// Vectors a thread holds between the min / max sweep and the quantization when its row is a
// whole number of 16-byte vectors: rows of up to kBlock * kRowqHold vectors are read once.
constexpr int kRowqHold = 8;

__device__ inline bool vec_aligned(const void *p) { return ((uintptr_t)p & 15u) == 0; }

template <typename T>
__global__ __launch_bounds__(kBlock) void rowq_fwd_kernel(RowqBatch batch, float qmax)
{
    constexpr int VEC = T::VEC;
    using vec_t = typename T::vec_t;
    __shared__ float part[2][kBlock / kWave];
    const int64_t b = blockIdx.x;
    const int i = find_item(batch.first_row, batch.count, b);
    const granq_rowq_item_t it = batch.item[i];
    const int64_t row = b - batch.first_row[i];
    const int64_t base = row * it.row_len;
    // block-uniform: 16-byte accesses need whole vectors per row and aligned tensors
    const bool vector = it.row_len % VEC == 0 && vec_aligned(it.w) && vec_aligned(it.w_hat);
    const int64_t vecs = it.row_len / VEC;
    const bool held = vector && vecs <= (int64_t)kBlock * kRowqHold;

    float mn = __builtin_inff(), mx = -__builtin_inff();
    vec_t keep[kRowqHold];
    if (held) {
        const vec_t *src = (const vec_t *)it.w + base / VEC;
#pragma unroll
        for (int u = 0; u < kRowqHold; ++u)
            if (threadIdx.x + u * kBlock < vecs) keep[u] = src[threadIdx.x + u * kBlock];
#pragma unroll
        for (int u = 0; u < kRowqHold; ++u)
            if (threadIdx.x + u * kBlock < vecs) {
                float f[VEC];
                T::unpack(keep[u], f);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    mn = __builtin_fminf(mn, f[e]);
                    mx = __builtin_fmaxf(mx, f[e]);
                }
            }
    } else if (vector) {
        const vec_t *src = (const vec_t *)it.w + base / VEC;
        for (int64_t k = threadIdx.x; k < vecs; k += kBlock) {
            float f[VEC];
            T::unpack(src[k], f);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                mn = __builtin_fminf(mn, f[e]);
                mx = __builtin_fmaxf(mx, f[e]);
            }
        }
    } else {
        for (int64_t k = threadIdx.x; k < it.row_len; k += kBlock) {
            const float v = T::load1(it.w, base + k);
            mn = __builtin_fminf(mn, v);
            mx = __builtin_fmaxf(mx, v);
        }
    }
    block_minmax(mn, mx, part);

    // Eq. 2, with the same degenerate-range rule as granq_prescale
    float s, z;
    channel_scale(mn, mx, qmax, s, z);
    if (threadIdx.x == 0) {
        it.scale[row] = s;
        it.zero_point[row] = z;
    }
    if (held) {
        vec_t *dst = (vec_t *)it.w_hat + base / VEC;
#pragma unroll
        for (int u = 0; u < kRowqHold; ++u)
            if (threadIdx.x + u * kBlock < vecs) {
                float f[VEC];
                T::unpack(keep[u], f);
#pragma unroll
                for (int e = 0; e < VEC; ++e) f[e] = dequant(clamp_code(raw_code(f[e], s, z), qmax), s, z);
                dst[threadIdx.x + u * kBlock] = T::pack(f);
            }
    } else if (vector) {
        const vec_t *src = (const vec_t *)it.w + base / VEC;
        vec_t *dst = (vec_t *)it.w_hat + base / VEC;
        for (int64_t k = threadIdx.x; k < vecs; k += kBlock) {
            float f[VEC];
            T::unpack(src[k], f);
#pragma unroll
            for (int e = 0; e < VEC; ++e) f[e] = dequant(clamp_code(raw_code(f[e], s, z), qmax), s, z);
            dst[k] = T::pack(f);
        }
    } else {
        for (int64_t k = threadIdx.x; k < it.row_len; k += kBlock) {
            const float q = clamp_code(raw_code(T::load1(it.w, base + k), s, z), qmax);
            T::store1(it.w_hat, base + k, dequant(q, s, z));
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void rowq_bwd_kernel(RowqBwdBatch batch, float qmax)
{
    constexpr int VEC = T::VEC;
    using vec_t = typename T::vec_t;
    const int64_t b = blockIdx.x;
    const int i = find_item(batch.first_row, batch.count, b);
    const granq_rowq_bwd_item_t it = batch.item[i];
    const int64_t row = b - batch.first_row[i];
    const int64_t base = row * it.row_len;
    const float s = it.scale[row], z = it.zero_point[row];
    if (it.row_len % VEC == 0 && vec_aligned(it.w) && vec_aligned(it.dy) && vec_aligned(it.dw)) {
        const vec_t *src = (const vec_t *)it.w + base / VEC;
        const vec_t *grad = (const vec_t *)it.dy + base / VEC;
        vec_t *dst = (vec_t *)it.dw + base / VEC;
        for (int64_t k = threadIdx.x; k < it.row_len / VEC; k += kBlock) {
            float f[VEC];
            bool keep[VEC];
            const vec_t g = grad[k];
            T::unpack(src[k], f);
#pragma unroll
            for (int e = 0; e < VEC; ++e) keep[e] = in_range(raw_code(f[e], s, z), qmax);
            dst[k] = T::gate(g, keep);
        }
        return;
    }
    for (int64_t k = threadIdx.x; k < it.row_len; k += kBlock) {
        const bool keep = in_range(raw_code(T::load1(it.w, base + k), s, z), qmax);
        T::store_gated1(it.dw, it.dy, base + k, keep);
    }
}

static bool elem_aligned(const void *p, granq_dtype_t dt) {
    return ((uintptr_t)p & (dt == GRANQ_F32 ? 3u : 1u)) == 0;
}

}  // namespace granq

using namespace granq;

extern "C" {

granq_status_t granq_rowwise_fakequant_multi(const granq_rowq_item_t *items, int count,
                                             granq_dtype_t dtype, int bits, void *stream) {
    if (!items || count <= 0) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (dtype != GRANQ_F32 && dtype != GRANQ_BF16 && dtype != GRANQ_F16) return GRANQ_ERR_UNSUPPORTED;
    for (int i = 0; i < count; ++i) {
        const granq_rowq_item_t &it = items[i];
        if (!it.w || !it.w_hat || !it.scale || !it.zero_point) return GRANQ_ERR_INVALID_ARG;
        if (it.rows <= 0 || it.row_len <= 0) return GRANQ_ERR_INVALID_ARG;
        if (it.rows >= ((int64_t)1 << 30) || it.row_len >= ((int64_t)1 << 40)) return GRANQ_ERR_UNSUPPORTED;
        if (!elem_aligned(it.w, dtype) || !elem_aligned(it.w_hat, dtype) ||
            !elem_aligned(it.scale, GRANQ_F32) || !elem_aligned(it.zero_point, GRANQ_F32))
            return GRANQ_ERR_UNSUPPORTED;
    }
    const float qmax = (float)((1 << bits) - 1);
    for (int at = 0; at < count; at += kMaxItems) {
        RowqBatch batch;
        batch.count = count - at < kMaxItems ? count - at : kMaxItems;
        int64_t rows = 0;
        for (int i = 0; i < batch.count; ++i) {
            batch.item[i] = items[at + i];
            batch.first_row[i] = rows;
            rows += items[at + i].rows;
        }
        for (int i = batch.count; i <= kMaxItems; ++i) batch.first_row[i] = rows;
        if (rows >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
        if (dtype == GRANQ_F32)
            launch_kernel(rowq_fwd_kernel<F32>, dim3((uint32_t)rows), dim3(kBlock), 0, (hipStream_t)stream, batch, qmax);
        else if (dtype == GRANQ_BF16)
            launch_kernel(rowq_fwd_kernel<BF16>, dim3((uint32_t)rows), dim3(kBlock), 0, (hipStream_t)stream, batch, qmax);
        else
            launch_kernel(rowq_fwd_kernel<F16>, dim3((uint32_t)rows), dim3(kBlock), 0, (hipStream_t)stream, batch, qmax);
        if (launched() != GRANQ_OK) return GRANQ_ERR_HIP;
    }
    return GRANQ_OK;
}

granq_status_t granq_rowwise_fakequant_bwd_multi(const granq_rowq_bwd_item_t *items, int count,
                                                 granq_dtype_t dtype, int bits, void *stream) {
    if (!items || count <= 0) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (dtype != GRANQ_F32 && dtype != GRANQ_BF16 && dtype != GRANQ_F16) return GRANQ_ERR_UNSUPPORTED;
    for (int i = 0; i < count; ++i) {
        const granq_rowq_bwd_item_t &it = items[i];
        if (!it.w || !it.dy || !it.dw || !it.scale || !it.zero_point) return GRANQ_ERR_INVALID_ARG;
        if (it.rows <= 0 || it.row_len <= 0) return GRANQ_ERR_INVALID_ARG;
        if (it.rows >= ((int64_t)1 << 30) || it.row_len >= ((int64_t)1 << 40)) return GRANQ_ERR_UNSUPPORTED;
        if (!elem_aligned(it.w, dtype) || !elem_aligned(it.dy, dtype) || !elem_aligned(it.dw, dtype) ||
            !elem_aligned(it.scale, GRANQ_F32) || !elem_aligned(it.zero_point, GRANQ_F32))
            return GRANQ_ERR_UNSUPPORTED;
    }
    const float qmax = (float)((1 << bits) - 1);
    for (int at = 0; at < count; at += kMaxItems) {
        RowqBwdBatch batch;
        batch.count = count - at < kMaxItems ? count - at : kMaxItems;
        int64_t rows = 0;
        for (int i = 0; i < batch.count; ++i) {
            batch.item[i] = items[at + i];
            batch.first_row[i] = rows;
            rows += items[at + i].rows;
        }
        for (int i = batch.count; i <= kMaxItems; ++i) batch.first_row[i] = rows;
        if (rows >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
        if (dtype == GRANQ_F32)
            launch_kernel(rowq_bwd_kernel<F32>, dim3((uint32_t)rows), dim3(kBlock), 0, (hipStream_t)stream, batch, qmax);
        else if (dtype == GRANQ_BF16)
            launch_kernel(rowq_bwd_kernel<BF16>, dim3((uint32_t)rows), dim3(kBlock), 0, (hipStream_t)stream, batch, qmax);
        else
            launch_kernel(rowq_bwd_kernel<F16>, dim3((uint32_t)rows), dim3(kBlock), 0, (hipStream_t)stream, batch, qmax);
        if (launched() != GRANQ_OK) return GRANQ_ERR_HIP;
    }
    return GRANQ_OK;
}

}  // extern "C"
