// Floating-point accumulation over the pre-scaled activations: the 1x1 convolution
//     y[n,o,k] = sum_c w[o,c] * x_hat[n,c,k]
// of Eq. 6 of the paper with a full weight matrix, beside the integer-domain form of
// granq_conv.hip.  Products and sums are binary32 on the matrix cores
// (v_mfma_f32_32x32x2_f32); 16-bit storage is widened on the load (exact) and narrowed on
// the store.
//
// Operand layout of the instruction (64 lanes, lane l):
//   A (32 x 2):  row l % 32, k = l / 32, one float
//   B (2 x 32):  column l % 32, k = l / 32, one float
//   D (32 x 32): column l % 32, register r holds row 8 * (r / 4) + 4 * (l / 32) + r % 4
// x_hat is NCHW, so a lane's load of four neighbouring pixels of ONE channel (16 bytes) is
// four B operands as it stands: matrix instruction j of a step covers pixels 4 * (l % 32) + j,
// no transpose.  The order of the channels inside a group of eight is free as long as both
// operands agree: step s of a group pairs channel s (lanes 0-31) with channel 4 + s (lanes
// 32-63), so that a lane's weights of a whole group are four consecutive floats of its row.
// A wavefront owns 128 pixels x 64 output channels (128 accumulator registers); per group of
// eight channels it loads 4 + 2 vectors and issues 32 matrix instructions, so the loads of
// the next group hide behind the arithmetic of the current one and nothing is staged in LDS.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "granq.h"
#include "granq_device.h"
#include "granq_launch.h"
#include "granq_pixels.h"

namespace granq {

typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kFcDies = 8;                 // XCDs of the chip
#ifndef GRANQ_FC_TILES
#define GRANQ_FC_TILES 2
#endif
constexpr int kFcT = GRANQ_FC_TILES;       // 32-row tiles of output channels per wavefront
constexpr int kFcRows = 32 * kFcT;         // output channels per wavefront
constexpr int kFcGroup = 8;                // channels per group: four steps of two

__device__ __forceinline__ void widen2(BF16, uint32_t w, float &lo, float &hi) { lo = bf16_lo(w); hi = bf16_hi(w); }
__device__ __forceinline__ void widen2(F16, uint32_t w, float &lo, float &hi) { F16::unpack2(w, lo, hi); }

// Four neighbouring elements from element index `at`, as binary32.  ALIGNED: `at` is a multiple
// of 4 and the base is aligned to four elements; otherwise the access is aligned to one element.
template <typename T, bool ALIGNED>
__device__ __forceinline__ f32x4 load4(const void *p, int64_t at) {
    if constexpr (T::ESIZE == 4) {
        typedef float f32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));
        if constexpr (ALIGNED) return *(const f32x4 *)((const float *)p + at);
        else return *(const f32x4_a4 *)((const float *)p + at);
    } else {
        typedef uint32_t u32x2_a2 __attribute__((ext_vector_type(2), aligned(2)));
        u32x2 v;
        if constexpr (ALIGNED) v = *(const u32x2 *)((const uint16_t *)p + at);
        else v = *(const u32x2_a2 *)((const uint16_t *)p + at);
        float f0, f1, f2, f3;
        widen2(T{}, v.x, f0, f1);
        widen2(T{}, v.y, f2, f3);
        return (f32x4){f0, f1, f2, f3};
    }
}

// Blocks are numbered so that die d (workgroups go to the eight dies round-robin) takes the d-th
// eighth of the tasks: the wavefronts that share a pixel tile (its sweeps of 64 output channels)
// and the neighbouring tiles meet in one die's L2.
// RAGGED: H*W is not a multiple of 4.  A sample then has ceil(H*W / 4) groups of pixels, the
// accesses are aligned to one element, and the last group's vector is the LAST four elements of
// the channel's row moved down so that the group's `valid` pixels come first.
template <typename T, bool RAGGED>
__global__ __launch_bounds__(kBlock, 2) void fconv1x1_mfma(
    const void *__restrict__ x, const void *__restrict__ w, void *__restrict__ y, int64_t c, int64_t hw,
    int64_t o, int64_t groups_total, int64_t tasks, int32_t sweeps, int32_t blocks_per_die, int32_t stream_out)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int half = lane / 32, col = lane % 32;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const uint32_t die = blockIdx.x % kFcDies, m = blockIdx.x / kFcDies;
    const int64_t task = ((int64_t)die * blocks_per_die + m) * (kBlock / kWave) + wave;
    if (task >= tasks) return;                          // wave-uniform; the kernel has no barrier
    const int64_t tile = task / sweeps;
    const int64_t o_base = (task - tile * sweeps) * kFcRows;
    const int64_t g = tile * 32 + col;
    const bool live = g < groups_total;
    const int64_t hw4 = RAGGED ? (hw + 3) / 4 : hw / 4; // groups per sample
    const int64_t n = live ? g / hw4 : 0;
    const int64_t pb = live ? 4 * (g - n * hw4) : 0;
    const int valid = RAGGED && hw - pb < 4 ? (int)(hw - pb) : 4;
    const int64_t pl = valid == 4 ? pb : hw - 4;        // where the group's vector is fetched
    const int down = 4 - valid;                         // elements to move it down by
    // element index of this lane's pixels in channel 4 * half of its sample; a lane without a
    // group reads sample 0 and stores nothing
    const int64_t x_lane = (n * c + 4 * half) * hw + pl;
    // rows past O (O is a multiple of 32, the second tile may lie past it) are never stored
    int64_t w_lane[kFcT];
#pragma unroll
    for (int t = 0; t < kFcT; ++t) {
        const int64_t row = o_base + 32 * t + col < o ? o_base + 32 * t + col : o - 1;
        w_lane[t] = row * c + 4 * half;
    }

    f32x16 acc[kFcT][4];
#pragma unroll
    for (int t = 0; t < kFcT; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][j][r] = 0.0f;

    // operands of a group of eight channels: fa[t][s], fb[s][j]
    auto fetch = [&](int64_t c0, f32x4 (&fa)[kFcT], f32x4 (&fb)[4]) {
#pragma unroll
        for (int t = 0; t < kFcT; ++t) fa[t] = load4<T, true>(w, w_lane[t] + c0);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            f32x4 v = load4<T, !RAGGED>(x, x_lane + (c0 + s) * hw);
            if (RAGGED) {
                if (down & 1) v = (f32x4){v.y, v.z, v.w, 0.0f};
                if (down & 2) v = (f32x4){v.z, v.w, 0.0f, 0.0f};
            }
            fb[s] = v;
        }
    };
    auto multiply = [&](const f32x4 (&fa)[kFcT], const f32x4 (&fb)[4]) {
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int t = 0; t < kFcT; ++t)
                    acc[t][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[t][s], fb[s][j], acc[t][j], 0, 0, 0);
    };
    // The loads of the next group are requested before the matrix instructions of the current one
    // and waited for after them; the compute unit's other wavefronts fill the wait.  (Keeping two
    // register sets so that a group's loads have a whole group of arithmetic to arrive measured
    // slower: 467 against 297 us on 1024 -> 256 channels at 14 x 14, batch 256.)
    f32x4 a[kFcT], b[4];
    fetch(0, a, b);
    for (int64_t c0 = 0; c0 < c; c0 += kFcGroup) {
        f32x4 na[kFcT], nb[4];
        const bool more = c0 + kFcGroup < c;            // wave-uniform
        if (more) fetch(c0 + kFcGroup, na, nb);
        multiply(a, b);
        if (more) {
#pragma unroll
            for (int t = 0; t < kFcT; ++t) a[t] = na[t];
#pragma unroll
            for (int s = 0; s < 4; ++s) b[s] = nb[s];
        }
    }
    if (!live) return;
    auto epilogue = [&](auto stream) {
        constexpr bool kStream = decltype(stream)::value;
        if (!kStream) keep_apart();
#pragma unroll
        for (int t = 0; t < kFcT; ++t) {
            if (o_base + 32 * t >= o) break;            // wave-uniform
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t oc = o_base + 32 * t + 8 * (r / 4) + 4 * half + (r % 4);
                const f32x4 v = {acc[t][0][r], acc[t][1][r], acc[t][2][r], acc[t][3][r]};
                if constexpr (RAGGED) store_pixels_ragged<T, kStream>(y, (n * o + oc) * hw + pb, v, valid);
                else store_pixels4<T, kStream>(y, (n * o + oc) * hw + pb, v);
            }
        }
        if (!kStream) keep_apart();
    };
    if (stream_out) epilogue(Flag<true>{});
    else epilogue(Flag<false>{});
}

// 16-bit storage on the 16-bit matrix instruction (v_mfma_f32_32x32x16_bf16 / _f16: products of
// the stored values exact, sums binary32).  Operands: A row l % 32, B column l % 32, both the
// eight consecutive k starting at 8 * (l / 32), two per dword; D as above.  A lane loads, for its
// eight channels, four neighbouring pixels each (8 bytes) and transposes the 8 x 4 halfwords in
// registers (v_perm_b32) into four B operands; its weights of a step are 16 consecutive bytes of
// its row.  One step = sixteen channels; tiles, tasks and the ragged case as in the kernel above.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ f32x16 mfma16(BF16, const u32x4 &a, const u32x4 &b, const f32x16 &c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}
__device__ __forceinline__ f32x16 mfma16(F16, const u32x4 &a, const u32x4 &b, const f32x16 &c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

constexpr int kFc16Step = 16;              // channels per matrix step

template <typename T, bool RAGGED>
__global__ __launch_bounds__(kBlock, 2) void fconv1x1_mfma16(
    const void *__restrict__ x, const void *__restrict__ w, void *__restrict__ y, int64_t c, int64_t hw,
    int64_t o, int64_t groups_total, int64_t tasks, int32_t sweeps, int32_t blocks_per_die, int32_t stream_out)
{
    static_assert(T::ESIZE == 2, "16-bit storage");
    typedef uint32_t u32x2_a2 __attribute__((ext_vector_type(2), aligned(2)));
    const int lane = threadIdx.x & (kWave - 1);
    const int half = lane / 32, col = lane % 32;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    const uint32_t die = blockIdx.x % kFcDies, m = blockIdx.x / kFcDies;
    const int64_t task = ((int64_t)die * blocks_per_die + m) * (kBlock / kWave) + wave;
    if (task >= tasks) return;                          // wave-uniform; the kernel has no barrier
    const int64_t tile = task / sweeps;
    const int64_t o_base = (task - tile * sweeps) * kFcRows;
    const int64_t g = tile * 32 + col;
    const bool live = g < groups_total;
    const int64_t hw4 = RAGGED ? (hw + 3) / 4 : hw / 4;
    const int64_t n = live ? g / hw4 : 0;
    const int64_t pb = live ? 4 * (g - n * hw4) : 0;
    const int valid = RAGGED && hw - pb < 4 ? (int)(hw - pb) : 4;
    const int64_t pl = valid == 4 ? pb : hw - 4;
    const int down = 16 * (4 - valid);                  // bits to move the last group's vector down by
    const uint16_t *xp = (const uint16_t *)x + (n * c + 8 * half) * hw + pl;
    const uint16_t *wp[kFcT];
#pragma unroll
    for (int t = 0; t < kFcT; ++t) {
        const int64_t row = o_base + 32 * t + col < o ? o_base + 32 * t + col : o - 1;
        wp[t] = (const uint16_t *)w + row * c + 8 * half;
    }

    f32x16 acc[kFcT][4];
#pragma unroll
    for (int t = 0; t < kFcT; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][j][r] = 0.0f;

    // a step's raw loads: the weights as they are, the lane's eight channels x four pixels
    auto fetch = [&](int64_t c0, u32x4 (&fa)[kFcT], u32x2 (&fd)[8]) {
#pragma unroll
        for (int t = 0; t < kFcT; ++t) fa[t] = *(const u32x4 *)(wp[t] + c0);
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (RAGGED) fd[i] = *(const u32x2_a2 *)(xp + (c0 + i) * hw);
            else fd[i] = *(const u32x2 *)(xp + (c0 + i) * hw);
        }
    };
    auto multiply = [&](const u32x4 (&fa)[kFcT], const u32x2 (&fd)[8]) {
        u32x4 b[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32x2 d0 = fd[2 * q], d1 = fd[2 * q + 1];
            if (RAGGED) {
                const uint64_t s0 = (((uint64_t)d0.y << 32) | d0.x) >> down, s1 = (((uint64_t)d1.y << 32) | d1.x) >> down;
                d0 = (u32x2){(uint32_t)s0, (uint32_t)(s0 >> 32)};
                d1 = (u32x2){(uint32_t)s1, (uint32_t)(s1 >> 32)};
            }
            // v_perm_b32(hi, lo, sel): selector bytes 0..3 pick bytes of lo, 4..7 bytes of hi
            b[0][q] = __builtin_amdgcn_perm(d1.x, d0.x, 0x05040100u);   // pixel 0 of channels 2q, 2q + 1
            b[1][q] = __builtin_amdgcn_perm(d1.x, d0.x, 0x07060302u);   // pixel 1
            b[2][q] = __builtin_amdgcn_perm(d1.y, d0.y, 0x05040100u);   // pixel 2
            b[3][q] = __builtin_amdgcn_perm(d1.y, d0.y, 0x07060302u);   // pixel 3
        }
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int t = 0; t < kFcT; ++t) acc[t][j] = mfma16(T{}, fa[t], b[j], acc[t][j]);
    };
    u32x4 a[kFcT];
    u32x2 d[8];
    fetch(0, a, d);
    for (int64_t c0 = 0; c0 < c; c0 += kFc16Step) {
        u32x4 na[kFcT];
        u32x2 nd[8];
        const bool more = c0 + kFc16Step < c;           // wave-uniform
        if (more) fetch(c0 + kFc16Step, na, nd);
        multiply(a, d);
        if (more) {
#pragma unroll
            for (int t = 0; t < kFcT; ++t) a[t] = na[t];
#pragma unroll
            for (int i = 0; i < 8; ++i) d[i] = nd[i];
        }
    }
    if (!live) return;
    auto epilogue = [&](auto stream) {
        constexpr bool kStream = decltype(stream)::value;
        if (!kStream) keep_apart();
#pragma unroll
        for (int t = 0; t < kFcT; ++t) {
            if (o_base + 32 * t >= o) break;            // wave-uniform
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t oc = o_base + 32 * t + 8 * (r / 4) + 4 * half + (r % 4);
                const f32x4 v = {acc[t][0][r], acc[t][1][r], acc[t][2][r], acc[t][3][r]};
                if constexpr (RAGGED) store_pixels_ragged<T, kStream>(y, (n * o + oc) * hw + pb, v, valid);
                else store_pixels4<T, kStream>(y, (n * o + oc) * hw + pb, v);
            }
        }
        if (!kStream) keep_apart();
    };
    if (stream_out) epilogue(Flag<true>{});
    else epilogue(Flag<false>{});
}

// Any shape: one thread per output element, binary32 multiply and add in channel order.
template <typename T>
__global__ __launch_bounds__(kBlock) void fconv1x1_plain(
    const void *__restrict__ x, const void *__restrict__ w, void *__restrict__ y, int64_t c, int64_t hw, int64_t o)
{
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t oc = blockIdx.y;
    const int64_t n = blockIdx.z;
    if (k >= hw) return;
    float acc = 0.0f;
    for (int64_t ic = 0; ic < c; ++ic) {
        const float term = T::load1(w, oc * c + ic) * T::load1(x, (n * c + ic) * hw + k);
        acc = acc + term;
    }
    T::store1(y, (n * o + oc) * hw + k, acc);
}

}  // namespace granq

using namespace granq;

typedef void (*fconv_mfma_t)(const void *, const void *, void *, int64_t, int64_t, int64_t, int64_t, int64_t,
                             int32_t, int32_t, int32_t);
typedef void (*fconv_plain_t)(const void *, const void *, void *, int64_t, int64_t, int64_t);

// 16-bit storage: the 16-bit matrix instruction when C is a multiple of 16 (and the eight weights
// of a lane are 16-byte aligned), else the binary32 one on widened values
template <bool RAGGED>
static fconv_mfma_t fconv_mfma_kernel(granq_dtype_t t, bool sixteen) {
    if (t == GRANQ_F32) return fconv1x1_mfma<F32, RAGGED>;
    if (t == GRANQ_BF16) return sixteen ? fconv1x1_mfma16<BF16, RAGGED> : fconv1x1_mfma<BF16, RAGGED>;
    return sixteen ? fconv1x1_mfma16<F16, RAGGED> : fconv1x1_mfma<F16, RAGGED>;
}

extern "C" granq_status_t granq_conv1x1_float(const void *x_hat, const granq_desc_t *desc, int64_t o,
                                              const void *w, void *y, void *stream) {
    if (!desc || !x_hat || !w || !y) return GRANQ_ERR_INVALID_ARG;
    if (desc->n <= 0 || desc->c <= 0 || desc->h <= 0 || desc->w <= 0 || o <= 0) return GRANQ_ERR_INVALID_ARG;
    const granq_dtype_t t = desc->dtype;
    if (t != GRANQ_F32 && t != GRANQ_BF16 && t != GRANQ_F16) return GRANQ_ERR_INVALID_ARG;
    const int64_t c = desc->c, hw = desc->h * desc->w, n = desc->n;
    if (o >= 65536 || n >= 65536 || c >= ((int64_t)1 << 24) || hw >= ((int64_t)1 << 36)) return GRANQ_ERR_UNSUPPORTED;
    const uintptr_t esize = t == GRANQ_F32 ? 4 : 2;
    if (((uintptr_t)x_hat & (esize - 1)) || ((uintptr_t)w & (esize - 1)) || ((uintptr_t)y & (esize - 1)))
        return GRANQ_ERR_UNSUPPORTED;
    hipStream_t hs = (hipStream_t)stream;
    // a lane handles four neighbouring pixels of a sample and four consecutive weights of a row
    const bool ragged = hw % 4 != 0;
    const uintptr_t four = 4 * esize - 1;
    const bool mfma = c % kFcGroup == 0 && o % 32 == 0 && hw >= 4 && ((uintptr_t)w & four) == 0 &&
                      (ragged || (((uintptr_t)x_hat & four) == 0 && ((uintptr_t)y & four) == 0));
    if (mfma) {
        const int64_t groups_total = n * ((hw + 3) / 4);
        const int64_t tiles = (groups_total + 31) / 32;
        const int64_t sweeps = (o + kFcRows - 1) / kFcRows;
        const int64_t tasks = tiles * sweeps;
        const int64_t per_block = kBlock / kWave;
        const int64_t blocks_per_die = ((tasks + per_block - 1) / per_block + kFcDies - 1) / kFcDies;
        if (blocks_per_die * kFcDies >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
        dim3 grid((uint32_t)(blocks_per_die * kFcDies)), block(kBlock);
        const bool sixteen = esize == 2 && c % kFc16Step == 0 && ((uintptr_t)w & 15u) == 0;
        fconv_mfma_t kernel = ragged ? fconv_mfma_kernel<true>(t, sixteen) : fconv_mfma_kernel<false>(t, sixteen);
        launch_kernel(kernel, grid, block, 0, hs, x_hat, w, y, c, hw, o, groups_total, tasks, (int32_t)sweeps,
                      (int32_t)blocks_per_die, (int32_t)(n * o * hw * (int64_t)esize > GRANQ_CONV_STREAM_OUT_BYTES));
        return launched();
    }
    if ((hw + kBlock - 1) / kBlock >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
    dim3 grid((uint32_t)((hw + kBlock - 1) / kBlock), (uint32_t)o, (uint32_t)n), block(kBlock);
    fconv_plain_t plain = t == GRANQ_F32 ? fconv1x1_plain<F32> : (t == GRANQ_BF16 ? fconv1x1_plain<BF16> : fconv1x1_plain<F16>);
    launch_kernel(plain, grid, block, 0, hs, x_hat, w, y, c, hw, o);
    return launched();
}
