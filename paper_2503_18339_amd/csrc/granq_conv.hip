// Integer-domain accumulation on the matrix cores: the 1x1 convolution that
// consumes the quantized activations, from their integer codes (Eq. 3 of the
// paper with w_c * s_c folded into int8 weights and the zero-point term summed
// once per output channel).
//
// Per sample the product is  D[O x HW] = Wq[O x C] . code[C x HW], int8 x int8 ->
// int32 with v_mfma_i32_32x32x32_i8.  Operand layout of the instruction (64 lanes,
// lane l; checked on the device against an integer matrix product):
//   A (32 x 32): row l % 32, sixteen consecutive k starting at 16 * (l / 32), one byte each
//   B (32 x 32): column l % 32, the same sixteen k
//   D (32 x 32): column l % 32, register r holds row 8 * (r / 4) + 4 * (l / 32) + r % 4
// The codes are NCHW, so consecutive k (channels) of one pixel are H*W bytes
// apart: a lane loads, for its sixteen channels, one dword (four neighbouring
// pixels) each and transposes the 16 x 4 bytes in registers (v_perm_b32) into
// four B operands; MFMA j of a group therefore covers pixels 4 * (l % 32) + j,
// and a lane ends up with four neighbouring pixels of every output row: one
// 16-byte store per row.  The weights of the block's 64 output channels are
// staged in LDS and shared by its four wavefronts.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "granq.h"
#include "granq_device.h"
#include "granq_launch.h"
#include "granq_pixels.h"

namespace granq {

typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));

constexpr int kConvOT = 2;                 // 32-channel output tiles per sweep
constexpr int kConvRows = 32 * kConvOT;    // output channels per sweep


constexpr int kConvKChunk = 512;           // channels staged in LDS at a time
#ifndef GRANQ_CONV_TARGET_BLOCKS
#define GRANQ_CONV_TARGET_BLOCKS 6000
#endif
constexpr int kConvDies = 8;               // XCDs of the chip
// The shared-tile variant below is taken from this many output and input channels on.
#ifndef GRANQ_CONV_SHARED
#define GRANQ_CONV_SHARED 1
#endif
#ifndef GRANQ_CONV_SHARED_MIN_O
#define GRANQ_CONV_SHARED_MIN_O 192
#endif
#ifndef GRANQ_CONV_SHARED_MIN_C
#define GRANQ_CONV_SHARED_MIN_C 128
#endif
constexpr int kConvPad = 16;               // bytes between LDS rows: 16-byte reads of 32 rows spread over all banks

// dword i of `d` holds four neighbouring pixels of channel i; the result's dword q of
// operand j holds channels 4q .. 4q+3 of pixel j.
__device__ __forceinline__ void transpose_16x4(const uint32_t (&d)[16], i32x4 (&b)[4]) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const uint32_t d0 = d[4 * q], d1 = d[4 * q + 1], d2 = d[4 * q + 2], d3 = d[4 * q + 3];
        // v_perm_b32(hi, lo, sel): selector bytes 0..3 pick bytes of lo, 4..7 bytes of hi
        const uint32_t p01 = __builtin_amdgcn_perm(d1, d0, 0x05010400u);   // pixels 0,1 of channels 0,1
        const uint32_t q01 = __builtin_amdgcn_perm(d1, d0, 0x07030602u);   // pixels 2,3 of channels 0,1
        const uint32_t p23 = __builtin_amdgcn_perm(d3, d2, 0x05010400u);
        const uint32_t q23 = __builtin_amdgcn_perm(d3, d2, 0x07030602u);
        b[0][q] = (int)__builtin_amdgcn_perm(p23, p01, 0x05040100u);
        b[1][q] = (int)__builtin_amdgcn_perm(p23, p01, 0x07060302u);
        b[2][q] = (int)__builtin_amdgcn_perm(q23, q01, 0x05040100u);
        b[3][q] = (int)__builtin_amdgcn_perm(q23, q01, 0x07060302u);
    }
}

// A wavefront owns 128 pixels (32 groups of four neighbouring pixels of one sample;
// groups are numbered through the whole batch, so only the batch's last wavefront
// is ragged); a block's four wavefronts share a range of "sweeps" of 64 output
// channels.  The sweeps are split over several blocks when the pixels alone do not
// give enough blocks to fill the chip; within a block the codes of later sweeps come
// from the caches.  Blocks are numbered so that the blocks that share a pixel tile
// (its `splits` groups of sweeps) are consecutive on ONE die: workgroups go to the
// eight dies round-robin in launch order and each die has its own L2, so the
// re-reads of a tile's codes by its other sweep groups hit that L2; die d takes the d-th eighth of
// the tiles, so that the cache lines a tile shares with its neighbours (a channel's row rarely
// starts on a line) are fetched by one die only.  The channel loop is software-pipelined by
// hand: the loads of the next 32 channels are issued before the matrix instructions of the
// current ones, and scheduling barriers keep them there.
// OutT: storage of y (F32, BF16 or F16 traits): the binary32 result is narrowed on the store.
// PACKED: the codes are two per byte; a lane then fetches its four pixels of a channel as one
// 16-bit load and spreads the nibbles into bytes (six integer operations) before the transpose.
// RAGGED: H*W is not a multiple of 4 (7 x 7 maps), codes one per byte.  A sample then has
// ceil(H*W / 4) groups; the dwords are fetched from addresses aligned to one byte; the last
// group's dword is the LAST four bytes of the channel's row, shifted down so that the group's
// `valid` pixels sit in the low bytes (above them stand codes of pixels that are never stored).
template <typename OutT, bool PACKED, bool RAGGED>
__global__ __launch_bounds__(kBlock, 2) void conv1x1_i8_mfma(
    const uint8_t *__restrict__ codes, const int8_t *__restrict__ wq, const int64_t *__restrict__ corr,
    const float *__restrict__ out_scale, void *__restrict__ y, int64_t c, int64_t hw, int64_t o,
    int64_t groups_total, int32_t sweeps_per_block, int32_t splits, int32_t lds_stride, int32_t tiles_per_die, int32_t stream_out)
{
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_w[];   // kConvRows x lds_stride bytes
    const int lane = threadIdx.x & (kWave - 1);
    const int half = lane / 32, col = lane % 32;
    // the wavefront's index, in a scalar register: everything derived from it is wave-uniform
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    // launch order -> (pixel tile, sweep group): die = id % 8, then the sweep groups of a tile
    const uint32_t die = blockIdx.x % kConvDies, m = blockIdx.x / kConvDies;
    const uint32_t split = m % (uint32_t)splits;
    const int64_t tile = (int64_t)die * tiles_per_die + m / (uint32_t)splits;
    const int64_t g_first = (tile * (kBlock / kWave) + wave) * 32;
    const int64_t g = g_first + col;
    const bool live = g < groups_total;
    const bool wave_live = __any(live);                // a dead wavefront only keeps the barriers
    static_assert(!(PACKED && RAGGED), "two codes per byte need H*W to be a multiple of 4");
    const int64_t hw4 = RAGGED ? (hw + 3) / 4 : hw / 4;   // groups per sample
    const int64_t n = live ? g / hw4 : 0;
    const int64_t pb = live ? 4 * (g - n * hw4) : 0;
    const int valid = RAGGED && hw - pb < 4 ? (int)(hw - pb) : 4;
    const int64_t pl = valid == 4 ? pb : hw - 4;        // where the group's dword is fetched
    const uint32_t shift = 8u * (uint32_t)(4 - valid);
    // addresses of the codes = wave-uniform base (scalar registers) + one 32-bit lane offset:
    // the wavefront's lanes lie within 33 samples of its first lane's sample (C*H*W < 2^25 here)
    const int64_t n_first = g_first < groups_total ? g_first / hw4 : 0;
    // raw buffer over the codes from the wavefront's first sample on: loads take the form
    // resource (scalar) + channel offset (scalar) + lane offset (one vector register)
    // (two codes per byte: every offset below is even, since hw is a multiple of 4)
    constexpr int kPerByte = PACKED ? 2 : 1;
    const __amdgpu_buffer_rsrc_t code_buf = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(codes + n_first * c * hw / kPerByte), 0, 0x7fffffff, 0x00020000);
    const uint32_t lane_off = live ? (uint32_t)(((n - n_first) * c * hw + pl + 16 * half * hw) / kPerByte) : 0u;

    const int64_t sweeps = (o + kConvRows - 1) / kConvRows;
    const int64_t s0 = (int64_t)split * sweeps_per_block;
    const int64_t s1 = s0 + sweeps_per_block < sweeps ? s0 + sweeps_per_block : sweeps;

    for (int64_t sw = s0; sw < s1; ++sw) {
        const int64_t o_base = sw * kConvRows;
        i32x16 acc[kConvOT][4];
#pragma unroll
        for (int t = 0; t < kConvOT; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][j][r] = 0;

        for (int64_t kc0 = 0; kc0 < c; kc0 += kConvKChunk) {
            const int32_t kcn = (int32_t)(c - kc0 < kConvKChunk ? c - kc0 : kConvKChunk);   // multiple of 16
            const int32_t kcr = (kcn + 63) / 64 * 64;  // the channel loop takes two 32-channel steps at a time
            __syncthreads();                           // the previous chunk's readers are done
            // stage Wq[o_base .. o_base+63][kc0 .. kc0+kcn) in 16-byte segments; rows past O and
            // channels past C read as zero
            const int32_t segs = kcr / 16;
            for (int32_t idx = threadIdx.x; idx < kConvRows * segs; idx += kBlock) {
                const int32_t row = idx / segs, seg = idx - row * segs;
                i32x4 v = {0, 0, 0, 0};
                if (o_base + row < o && seg * 16 < kcn)
                    v = *(const i32x4 *)(wq + (o_base + row) * c + kc0 + seg * 16);
                *(i32x4 *)(lds_w + row * lds_stride + seg * 16) = v;
            }
            __syncthreads();
            if (!wave_live) continue;

            const uint8_t *a_row0 = lds_w + col * lds_stride + 16 * half;
            const uint8_t *a_row1 = lds_w + (32 + col) * lds_stride + 16 * half;
            uint32_t d0[16], d1[16];
            // Issue the loads of this lane's sixteen channels of the 32-channel step at chunk
            // offset k.  Every lane loads, always: a lane or step without work (ragged last
            // wavefront, channels past C) reads in-bounds bytes that the multiply discards, so
            // the loop body is free of branches and the loads stay in flight across it.
#define GRANQ_CONV_FETCH(d, k)                                                              \
            {                                                                                \
                const int64_t ch0 = kc0 + (k);             /* wave-uniform */                \
                const bool ok = live && ch0 + 16 * half < c;                                 \
                const int off = (int)(ok ? lane_off : 0u);                                   \
                const int64_t ch0c = ch0 < c - 16 ? ch0 : c - 16;                            \
                _Pragma("unroll") for (int i = 0; i < 16; ++i)                               \
                    d[i] = PACKED ? (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(    \
                                        code_buf, off, (int)((ch0c + i) * hw / 2), 0)        \
                                  : (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(          \
                                        code_buf, off, (int)((ch0c + i) * hw), 0);           \
            }
#define GRANQ_CONV_MULTIPLY(d, k)                                                            \
            {                                                                                \
                const bool ok = live && kc0 + (k) + 16 * half < c;                           \
                _Pragma("unroll") for (int i = 0; i < 16; ++i) {                             \
                    uint32_t t = ok ? d[i] : 0u;                                             \
                    if (RAGGED) t >>= shift;                                                 \
                    if (PACKED) {                      /* nibble i -> byte i */              \
                        t = (t | (t << 8)) & 0x00FF00FFu;                                    \
                        t = (t | (t << 4)) & 0x0F0F0F0Fu;                                    \
                    }                                                                        \
                    d[i] = t;                                                                \
                }                                                                            \
                i32x4 b[4];                                                                  \
                transpose_16x4(d, b);                                                        \
                const i32x4 a0 = *(const i32x4 *)(a_row0 + (k));                             \
                _Pragma("unroll") for (int j = 0; j < 4; ++j)                                \
                    acc[0][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, b[j], acc[0][j], 0, 0, 0); \
                const i32x4 a1 = *(const i32x4 *)(a_row1 + (k));                             \
                _Pragma("unroll") for (int j = 0; j < 4; ++j)                                \
                    acc[1][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, b[j], acc[1][j], 0, 0, 0); \
            }
            // the scheduling barriers keep each batch of loads ahead of the multiply before it
            GRANQ_CONV_FETCH(d0, 0)
            for (int32_t k = 0; k < kcr; k += 64) {
                GRANQ_CONV_FETCH(d1, k + 32)
                __builtin_amdgcn_sched_barrier(0);
                GRANQ_CONV_MULTIPLY(d0, k)
                __builtin_amdgcn_sched_barrier(0);
                GRANQ_CONV_FETCH(d0, k + 64)               // past the chunk in the last round: discarded
                __builtin_amdgcn_sched_barrier(0);
                GRANQ_CONV_MULTIPLY(d1, k + 32)
                __builtin_amdgcn_sched_barrier(0);
            }
#undef GRANQ_CONV_FETCH
#undef GRANQ_CONV_MULTIPLY
        }
        if (!live) continue;
        auto epilogue = [&](auto stream) {
            constexpr bool kStream = decltype(stream)::value;
            if (!kStream) keep_apart();
#pragma unroll
            for (int t = 0; t < kConvOT; ++t) {
                if (o_base + 32 * t >= o) break;       // wave-uniform: o is a multiple of 32
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t oc = o_base + 32 * t + 8 * (r / 4) + 4 * half + (r % 4);
                    // the difference is exact in binary64 (|corr| < 2^48), so narrowing it rounds once:
                    // the same value as the conversion of the 64-bit integer difference
                    const double cz = (double)corr[oc];
                    const float sc = out_scale[oc];
                    f32x4 v;
                    v.x = sc * (float)((double)acc[t][0][r] - cz);
                    v.y = sc * (float)((double)acc[t][1][r] - cz);
                    v.z = sc * (float)((double)acc[t][2][r] - cz);
                    v.w = sc * (float)((double)acc[t][3][r] - cz);
                    if constexpr (RAGGED) store_pixels_ragged<OutT, kStream>(y, (n * o + oc) * hw + pb, v, valid);
                    else store_pixels4<OutT, kStream>(y, (n * o + oc) * hw + pb, v);
                }
            }
            if (!kStream) keep_apart();
        };
        if (stream_out) epilogue(Flag<true>{});
        else epilogue(Flag<false>{});
    }
}

// Variant for many output channels and many input channels (the weight-heavy 1x1 convolutions
// of the later stages): the four wavefronts of a block work on the SAME 128 pixels, each on
// its own 64 of 256 output channels, and share the transposed code tiles through LDS, so the
// codes are fetched and transposed once per 256 output channels instead of once per 64.
// Channels go in chunks of 128 (four 32-channel steps; 256 with two blocks' worth of LDS measured
// slower: 52 against 39 us on 1024 -> 256 channels at 14 x 14, batch 256): wavefront w fetches and
// transposes step w (w + 4, ... with longer chunks) and writes its four B operands to LDS in exactly
// the lane order in which every wavefront then reads them back; the chunk's weights (256 rows x 128
// bytes) are staged beside them.  The fetches of the next chunk (codes and weights, into registers)
// are in flight during the multiplies of the current one.
#ifndef GRANQ_CONV_SHARED_CHUNK
#define GRANQ_CONV_SHARED_CHUNK 128
#endif
constexpr int kShChunk = GRANQ_CONV_SHARED_CHUNK;          // channels per chunk: a multiple of 128
constexpr int kShRows = 4 * kConvRows;         // output channels per block
constexpr int kShTile = kWave * 4 * 16;        // bytes of one step's four B operands (64 lanes x 4 x 16)
constexpr int kShSteps = kShChunk / 32;        // 32-channel steps per chunk
constexpr int kShMine = kShSteps / 4;          // steps a wavefront fetches and transposes per chunk

template <typename OutT, bool PACKED, bool RAGGED>
__global__ __launch_bounds__(kBlock, 2) void conv1x1_i8_mfma_shared(
    const uint8_t *__restrict__ codes, const int8_t *__restrict__ wq, const int64_t *__restrict__ corr,
    const float *__restrict__ out_scale, void *__restrict__ y, int64_t c, int64_t hw, int64_t o,
    int64_t groups_total, int32_t supers, int32_t tiles_per_die, int32_t stream_out)
{
    static_assert(kShChunk % 128 == 0, "four wavefronts share the steps of a chunk evenly");
    constexpr int kStride = kShChunk + kConvPad;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds_all[];
    uint8_t *lds_w = lds_all;                              // kShRows x kStride
    uint8_t *lds_b = lds_all + kShRows * kStride;          // kShSteps x kShTile
    const int lane = threadIdx.x & (kWave - 1);
    const int half = lane / 32, col = lane % 32;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    // launch order -> pixel tile: workgroups go to the eight dies round-robin, so die d takes the d-th
    // eighth of the tiles.  Neighbouring tiles then meet in ONE die's L2: a channel's row of H*W bytes
    // rarely starts on a cache line, so each 128-byte piece shares its first and last line with the
    // neighbouring tile's piece (with round-robin tiles every such line came from memory twice).
    const uint32_t die = blockIdx.x % kConvDies, m = blockIdx.x / kConvDies;
    const int64_t tile = (int64_t)die * tiles_per_die + m / (uint32_t)supers;
    const int64_t super = m % (uint32_t)supers;
    if (tile * 32 >= groups_total) return;                 // block-uniform: the last die's spare blocks
    const int64_t g_first = tile * 32;                     // all four wavefronts: the same 32 pixel groups
    const int64_t g = g_first + col;
    const bool live = g < groups_total;
    static_assert(!(PACKED && RAGGED), "two codes per byte need H*W to be a multiple of 4");
    const int64_t hw4 = RAGGED ? (hw + 3) / 4 : hw / 4;   // groups per sample
    const int64_t n = live ? g / hw4 : 0;
    const int64_t pb = live ? 4 * (g - n * hw4) : 0;
    const int valid = RAGGED && hw - pb < 4 ? (int)(hw - pb) : 4;
    const int64_t pl = valid == 4 ? pb : hw - 4;        // where the group's dword is fetched
    const uint32_t shift = 8u * (uint32_t)(4 - valid);
    const int64_t n_first = g_first / hw4;                 // g_first < groups_total from here on
    constexpr int kPerByte = PACKED ? 2 : 1;
    const __amdgpu_buffer_rsrc_t code_buf = __builtin_amdgcn_make_buffer_rsrc(
        (void *)(codes + n_first * c * hw / kPerByte), 0, 0x7fffffff, 0x00020000);
    const uint32_t lane_off = live ? (uint32_t)(((n - n_first) * c * hw + pl + 16 * half * hw) / kPerByte) : 0u;
    const int64_t o_base = super * kShRows + wave * kConvRows;       // this wavefront's 64 output channels

    i32x16 acc[kConvOT][4];
#pragma unroll
    for (int t = 0; t < kConvOT; ++t)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][j][r] = 0;

    // this wavefront's steps of the chunk that starts at channel kc: steps wave, wave + 4, ...
    uint32_t d[kShMine][16];
    auto fetch = [&](int64_t kc) {
#pragma unroll
        for (int m = 0; m < kShMine; ++m) {
            const int64_t ch0 = kc + 32 * (wave + 4 * m);
            const bool ok = live && ch0 + 16 * half < c;
            const int off = (int)(ok ? lane_off : 0u);
            const int64_t ch0c = ch0 < c - 16 ? ch0 : c - 16;      // in bounds; what it reads is discarded
#pragma unroll
            for (int i = 0; i < 16; ++i)
                d[m][i] = PACKED ? (uint32_t)(uint16_t)__builtin_amdgcn_raw_buffer_load_b16(code_buf, off, (int)((ch0c + i) * hw / 2), 0)
                                 : (uint32_t)__builtin_amdgcn_raw_buffer_load_b32(code_buf, off, (int)((ch0c + i) * hw), 0);
        }
    };
    // the chunk's weights, one 16-byte segment per thread and round: rows past O and channels past
    // C read as zero
    constexpr int kSegs = kShChunk / 16;                   // segments per row
    constexpr int kRounds = kShRows * kSegs / kBlock;      // segments per thread
    i32x4 wreg[kRounds];
    auto wload = [&](int64_t kc) {
#pragma unroll
        for (int q = 0; q < kRounds; ++q) {
            const int32_t idx = threadIdx.x + q * kBlock;
            const int32_t row = idx / kSegs, seg = idx - row * kSegs;
            i32x4 v = {0, 0, 0, 0};
            if (super * kShRows + row < o && kc + seg * 16 < c)
                v = *(const i32x4 *)(wq + (super * kShRows + row) * c + kc + seg * 16);
            wreg[q] = v;
        }
    };
    fetch(0);
    wload(0);
    for (int64_t kc0 = 0; kc0 < c; kc0 += kShChunk) {
        __syncthreads();                                   // the previous chunk's readers are done
#pragma unroll
        for (int q = 0; q < kRounds; ++q) {
            const int32_t idx = threadIdx.x + q * kBlock;
            const int32_t row = idx / kSegs, seg = idx - row * kSegs;
            *(i32x4 *)(lds_w + row * kStride + seg * 16) = wreg[q];
        }
        // this wavefront's steps: discard what lies past C or belongs to no pixel, transpose, publish
#pragma unroll
        for (int m = 0; m < kShMine; ++m) {
            const int step = wave + 4 * m;
            const bool ok = live && kc0 + 32 * step + 16 * half < c;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                uint32_t t = ok ? d[m][i] : 0u;
                if (RAGGED) t >>= shift;
                if (PACKED) {                              // nibble i -> byte i
                    t = (t | (t << 8)) & 0x00FF00FFu;
                    t = (t | (t << 4)) & 0x0F0F0F0Fu;
                }
                d[m][i] = t;
            }
            i32x4 b[4];
            transpose_16x4(d[m], b);
#pragma unroll
            for (int j = 0; j < 4; ++j) *(i32x4 *)(lds_b + step * kShTile + (j * kWave + lane) * 16) = b[j];
        }
        if (kc0 + kShChunk < c) {                          // in flight during the multiplies below
            fetch(kc0 + kShChunk);
            wload(kc0 + kShChunk);
        }
        __syncthreads();
#pragma unroll
        for (int s = 0; s < kShSteps; ++s) {
            if (kc0 + 32 * s >= c) break;                  // block-uniform
            const i32x4 a0 = *(const i32x4 *)(lds_w + (wave * kConvRows + col) * kStride + 32 * s + 16 * half);
            const i32x4 a1 = *(const i32x4 *)(lds_w + (wave * kConvRows + 32 + col) * kStride + 32 * s + 16 * half);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const i32x4 bj = *(const i32x4 *)(lds_b + s * kShTile + (j * kWave + lane) * 16);
                acc[0][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a0, bj, acc[0][j], 0, 0, 0);
                acc[1][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a1, bj, acc[1][j], 0, 0, 0);
            }
        }
    }
    if (!live) return;
    auto epilogue = [&](auto stream) {
        constexpr bool kStream = decltype(stream)::value;
        if (!kStream) keep_apart();
#pragma unroll
        for (int t = 0; t < kConvOT; ++t) {
            if (o_base + 32 * t >= o) break;               // wave-uniform: o is a multiple of 32
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t oc = o_base + 32 * t + 8 * (r / 4) + 4 * half + (r % 4);
                const double cz = (double)corr[oc];
                const float sc = out_scale[oc];
                f32x4 v;
                v.x = sc * (float)((double)acc[t][0][r] - cz);
                v.y = sc * (float)((double)acc[t][1][r] - cz);
                v.z = sc * (float)((double)acc[t][2][r] - cz);
                v.w = sc * (float)((double)acc[t][3][r] - cz);
                if constexpr (RAGGED) store_pixels_ragged<OutT, kStream>(y, (n * o + oc) * hw + pb, v, valid);
                else store_pixels4<OutT, kStream>(y, (n * o + oc) * hw + pb, v);
            }
        }
        if (!kStream) keep_apart();
    };
    if (stream_out) epilogue(Flag<true>{});
    else epilogue(Flag<false>{});
}

// Any shape: one thread per output element, integer loop over the channels.
// PACKED: the codes are two per byte (element i in nibble i & 1 of byte i >> 1).
template <typename OutT, bool PACKED>
__global__ __launch_bounds__(kBlock) void conv1x1_i8_plain(
    const uint8_t *__restrict__ codes, const int8_t *__restrict__ wq, const int64_t *__restrict__ corr,
    const float *__restrict__ out_scale, void *__restrict__ y, int64_t c, int64_t hw, int64_t o)
{
    const int64_t k = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t oc = blockIdx.y;
    const int64_t n = blockIdx.z;
    if (k >= hw) return;
    int64_t acc = 0;
    for (int64_t ic = 0; ic < c; ++ic) {
        const int64_t at = (n * c + ic) * hw + k;
        const int32_t code = PACKED ? ((codes[at >> 1] >> (4 * (at & 1))) & 15) : codes[at];
        acc += (int64_t)((int32_t)wq[oc * c + ic] * code);
    }
    OutT::store1(y, (n * o + oc) * hw + k, out_scale[oc] * (float)(acc - corr[oc]));
}

// One block per output channel: fold the activation scale into the weights and
// quantize the row to int8 (symmetric), sum the zero-point term.
__global__ __launch_bounds__(kBlock) void fold_weights_kernel(
    const float *__restrict__ w, const float *__restrict__ scale, const float *__restrict__ zero_point,
    int64_t c, int8_t *__restrict__ wq, int64_t *__restrict__ corr, float *__restrict__ out_scale)
{
    __shared__ float part[kBlock / kWave];
    __shared__ int64_t ipart[kBlock / kWave];
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
    int64_t cz = 0;                                    // exact: |wq| <= 127, |z| < 2^24, c < 2^16
    for (int64_t ic = threadIdx.x; ic < c; ic += kBlock) {
        const float ws = w[oc * c + ic] * scale[ic];
        float q = __builtin_rintf(ws / a);
        q = __builtin_fminf(__builtin_fmaxf(q, -127.0f), 127.0f);
        const int32_t qi = (int32_t)q;
        wq[oc * c + ic] = (int8_t)qi;
        cz += (int64_t)qi * (int64_t)zero_point[ic];
    }
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) cz += (int64_t)__shfl_xor((long long)cz, off, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) ipart[threadIdx.x / kWave] = cz;
    __syncthreads();
    if (threadIdx.x == 0) {
        int64_t t = 0;
        for (int i = 0; i < kBlock / kWave; ++i) t += ipart[i];
        corr[oc] = t;
        out_scale[oc] = a;
    }
}

}  // namespace granq

using namespace granq;

typedef void (*conv_shared_t)(const uint8_t *, const int8_t *, const int64_t *, const float *, void *, int64_t,
                              int64_t, int64_t, int64_t, int32_t, int32_t, int32_t);
typedef void (*conv_mfma_t)(const uint8_t *, const int8_t *, const int64_t *, const float *, void *, int64_t,
                            int64_t, int64_t, int64_t, int32_t, int32_t, int32_t, int32_t, int32_t);
typedef void (*conv_plain_t)(const uint8_t *, const int8_t *, const int64_t *, const float *, void *, int64_t,
                             int64_t, int64_t);

template <bool PACKED, bool RAGGED>
static conv_shared_t shared_kernel(granq_dtype_t t) {
    return t == GRANQ_F32 ? conv1x1_i8_mfma_shared<F32, PACKED, RAGGED>
                          : (t == GRANQ_BF16 ? conv1x1_i8_mfma_shared<BF16, PACKED, RAGGED>
                                             : conv1x1_i8_mfma_shared<F16, PACKED, RAGGED>);
}
template <bool PACKED, bool RAGGED>
static conv_mfma_t mfma_kernel(granq_dtype_t t) {
    return t == GRANQ_F32 ? conv1x1_i8_mfma<F32, PACKED, RAGGED>
                          : (t == GRANQ_BF16 ? conv1x1_i8_mfma<BF16, PACKED, RAGGED> : conv1x1_i8_mfma<F16, PACKED, RAGGED>);
}
template <bool PACKED>
static conv_plain_t plain_kernel(granq_dtype_t t) {
    return t == GRANQ_F32 ? conv1x1_i8_plain<F32, PACKED>
                          : (t == GRANQ_BF16 ? conv1x1_i8_plain<BF16, PACKED> : conv1x1_i8_plain<F16, PACKED>);
}

// y_dtype: storage of y; the binary32 result is narrowed (round to nearest even) on the store.
template <bool PACKED>
static granq_status_t conv_impl(const uint8_t *codes, const granq_desc_t *desc, int64_t o,
                                const int8_t *wq, const int64_t *corr, const float *out_scale,
                                int bits, granq_dtype_t y_dtype, void *y, void *stream) {
    if (!desc || !codes || !wq || !corr || !out_scale || !y) return GRANQ_ERR_INVALID_ARG;
    if (desc->n <= 0 || desc->c <= 0 || desc->h <= 0 || desc->w <= 0 || o <= 0) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > (PACKED ? 4 : 8)) return GRANQ_ERR_INVALID_ARG;
    if (y_dtype != GRANQ_F32 && y_dtype != GRANQ_BF16 && y_dtype != GRANQ_F16) return GRANQ_ERR_UNSUPPORTED;
    const int64_t c = desc->c, hw = desc->h * desc->w, n = desc->n;
    // |sum| <= 127 * 255 * C must stay inside int32
    if (c >= ((int64_t)1 << 16) || o >= 65536 || n >= 65536 || hw >= ((int64_t)1 << 40)) return GRANQ_ERR_UNSUPPORTED;
    const uintptr_t esize = y_dtype == GRANQ_F32 ? 4 : 2;
    if (((uintptr_t)corr & 7u) || ((uintptr_t)out_scale & 3u) || ((uintptr_t)y & (esize - 1))) return GRANQ_ERR_UNSUPPORTED;
    hipStream_t hs = (hipStream_t)stream;
    // a lane handles four neighbouring pixels of a sample at once: aligned when H*W is a multiple of
    // 4, else (codes one per byte only) with accesses aligned to one element
    const bool ragged = hw % 4 != 0;
    const bool shape_ok = bits <= 7 && c % 16 == 0 && o % 32 == 0 && c * hw < ((int64_t)1 << 25) && ((uintptr_t)wq & 15u) == 0;
    const bool mfma = shape_ok && (ragged ? !PACKED && hw >= 4
                                          : ((uintptr_t)codes & (PACKED ? 1u : 3u)) == 0 && ((uintptr_t)y & (4 * esize - 1)) == 0);
    const int64_t groups_total = n * ((hw + 3) / 4);
    const int32_t stream_out = n * o * hw * (int64_t)esize > GRANQ_CONV_STREAM_OUT_BYTES;
    // many output and input channels: four wavefronts share one pixel tile's transposed codes
    if (mfma && GRANQ_CONV_SHARED && o >= GRANQ_CONV_SHARED_MIN_O && c >= GRANQ_CONV_SHARED_MIN_C) {
        const int64_t tiles = (groups_total + 31) / 32;
        const int64_t supers = (o + kShRows - 1) / kShRows;
        const int64_t tiles_per_die = (tiles + kConvDies - 1) / kConvDies;
        const int64_t blocks = tiles_per_die * kConvDies * supers;
        if (blocks >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
        const size_t lds_bytes = (size_t)kShRows * (kShChunk + kConvPad) + (size_t)kShSteps * kShTile;
        dim3 grid((uint32_t)blocks), block(kBlock);
        conv_shared_t kernel;
        if constexpr (PACKED) kernel = shared_kernel<true, false>(y_dtype);
        else kernel = ragged ? shared_kernel<false, true>(y_dtype) : shared_kernel<false, false>(y_dtype);
        // more than the 64 KB of LDS a kernel gets without asking (a function attribute, no allocation)
        if (hipFuncSetAttribute((const void *)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_bytes) != hipSuccess)
            return GRANQ_ERR_HIP;
        launch_kernel(kernel, grid, block, lds_bytes, hs, codes, wq, corr, out_scale, y, c, hw, o, groups_total,
                      (int32_t)supers, (int32_t)tiles_per_die, stream_out);
        return launched();
    }
    if (mfma) {
        const int64_t gx = (groups_total + 32 * (kBlock / kWave) - 1) / (32 * (kBlock / kWave));
        if (gx >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
        const int64_t sweeps = (o + kConvRows - 1) / kConvRows;
        // split the sweeps over several blocks until the launch has about this many
        int64_t gy = (GRANQ_CONV_TARGET_BLOCKS + gx - 1) / gx;
        if (gy > sweeps) gy = sweeps;
        if (gy < 1) gy = 1;
        const int64_t spb = (sweeps + gy - 1) / gy;
        gy = (sweeps + spb - 1) / spb;
        const int64_t kc = c < kConvKChunk ? (c + 63) / 64 * 64 : kConvKChunk;
        const int32_t lds_stride = (int32_t)kc + kConvPad;
        const size_t lds_bytes = (size_t)kConvRows * lds_stride;
        // each die's range of tiles rounded up; blocks of tiles past the end find no live group
        const int64_t tiles_per_die = (gx + kConvDies - 1) / kConvDies;
        const int64_t blocks = tiles_per_die * kConvDies * gy;
        if (blocks >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
        dim3 grid((uint32_t)blocks), block(kBlock);
        conv_mfma_t kernel;
        if constexpr (PACKED) kernel = mfma_kernel<true, false>(y_dtype);
        else kernel = ragged ? mfma_kernel<false, true>(y_dtype) : mfma_kernel<false, false>(y_dtype);
        launch_kernel(kernel, grid, block, lds_bytes, hs, codes, wq, corr, out_scale, y, c, hw, o, groups_total,
                      (int32_t)spb, (int32_t)gy, lds_stride, (int32_t)tiles_per_die, stream_out);
        return launched();
    }
    dim3 grid((uint32_t)((hw + kBlock - 1) / kBlock), (uint32_t)o, (uint32_t)n), block(kBlock);
    launch_kernel(plain_kernel<PACKED>(y_dtype), grid, block, 0, hs, codes, wq, corr, out_scale, y, c, hw, o);
    return launched();
}

extern "C" {

granq_status_t granq_fold_weights(const float *w, const float *scale, const float *zero_point,
                                  int64_t o, int64_t c, int8_t *wq, int64_t *corr, float *out_scale,
                                  void *stream) {
    if (!w || !scale || !zero_point || !wq || !corr || !out_scale) return GRANQ_ERR_INVALID_ARG;
    if (o <= 0 || c <= 0) return GRANQ_ERR_INVALID_ARG;
    if (o >= ((int64_t)1 << 31) || c >= ((int64_t)1 << 16)) return GRANQ_ERR_UNSUPPORTED;
    if (((uintptr_t)w & 3u) || ((uintptr_t)scale & 3u) || ((uintptr_t)zero_point & 3u) ||
        ((uintptr_t)corr & 7u) || ((uintptr_t)out_scale & 3u))
        return GRANQ_ERR_UNSUPPORTED;
    launch_kernel(fold_weights_kernel, dim3((uint32_t)o), dim3(kBlock), 0, (hipStream_t)stream,
                       w, scale, zero_point, c, wq, corr, out_scale);
    return launched();
}

granq_status_t granq_conv1x1_int8(const uint8_t *codes, const granq_desc_t *desc, int64_t o,
                                  const int8_t *wq, const int64_t *corr, const float *out_scale,
                                  int bits, float *y, void *stream) {
    return conv_impl<false>(codes, desc, o, wq, corr, out_scale, bits, GRANQ_F32, y, stream);
}

granq_status_t granq_conv1x1_int8_as(const uint8_t *codes, const granq_desc_t *desc, int64_t o,
                                     const int8_t *wq, const int64_t *corr, const float *out_scale,
                                     int bits, granq_dtype_t y_dtype, void *y, void *stream) {
    return conv_impl<false>(codes, desc, o, wq, corr, out_scale, bits, y_dtype, y, stream);
}

granq_status_t granq_conv1x1_int8_packed4(const uint8_t *packed, const granq_desc_t *desc, int64_t o,
                                          const int8_t *wq, const int64_t *corr, const float *out_scale,
                                          int bits, granq_dtype_t y_dtype, void *y, void *stream) {
    return conv_impl<true>(packed, desc, o, wq, corr, out_scale, bits, y_dtype, y, stream);
}

}  // extern "C"
