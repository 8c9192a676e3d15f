// GranQ activation fake-quantizer: gfx950 kernels and the C ABI around them.
//
// Four operations, as in the paper's Alg. 1 up to (not including) the
// accumulation:
//   range_reduce   per-channel min / max over (n,h,w)          Eq. 4, Sec. 5.1
//   prescale       scale and zero-point vectors, all channels  Eq. 5
//   fakequant_fwd  quantize, clamp, dequantize                 Eq. 1, Eq. 6
//   fakequant_bwd  straight-through gate                       Sec. 2.1
//
// All of them are bound by HBM bandwidth, so the kernels are organised around
// memory traffic: each element is loaded once with a 128-bit load and stored
// once with a 128-bit store, and everything per-channel sits in registers (see
// granq_plan.h for the column-tile decomposition that makes this possible).
// Tensors whose rows are not a whole number of 16-byte vectors, or whose
// pointers are not 16-byte aligned, take element-wise kernels ("row" kernels:
// one wavefront per (n,c) slab, scale and zero-point wave-uniform).
#include <hip/hip_runtime.h>
#include <float.h>
#include <stdlib.h>
#include <type_traits>
#include <atomic>
#include <stdint.h>

#include "granq.h"
#include "granq_device.h"
#include "granq_launch.h"
#include "granq_plan.h"
#include "granq_tiling.h"
#include "granq_internal.h"
#include "granq_quotient.h"

namespace granq {

#ifndef GRANQ_R_UNROLL
#define GRANQ_R_UNROLL 8
#endif
// The forward walks the tensor from its end towards its start: it usually runs
// right after the reduction, whose most recently read (last) rows are the ones
// still held by the memory-side cache.
#ifndef GRANQ_FWD_REVERSE
#define GRANQ_FWD_REVERSE 1
#endif
// Non-temporal stores for outputs nobody re-reads soon (x_hat, dx, codes).
#ifndef GRANQ_NT_STORE
#define GRANQ_NT_STORE 1
#endif
// Five-operation exact quotient (granq_quotient.h) instead of the general division.
#ifndef GRANQ_FAST_QUOTIENT
#define GRANQ_FAST_QUOTIENT 1
#endif

template <bool NT, typename V>
__device__ inline V load_vec(const V *p) {
    if (NT) return __builtin_nontemporal_load(p);
    return *p;
}

template <typename V>
__device__ inline void store_vec(V *p, const V &v) {
#if GRANQ_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// What a lane keeps per channel while it walks down its rows.
struct ChanRegs {
    float s, z, r;       // scale, zero-point, RN(1/scale)
};

// Rounded, unclamped code of Eq. 1.  FAST: x / s through the per-channel
// reciprocal, bit-identical where it matters (see granq_quotient.h).
template <bool FAST>
__device__ inline float code_of(float x, const ChanRegs &c) {
    float t;
    if (FAST) t = quotient_fast(quotient_clamp(x), c.s, c.r);
    else t = x / c.s;
    float v = t + c.z;
    return __builtin_rintf(v);
}

// Eq. 5 for one channel: step size and zero-point from the channel's range.
__device__ __forceinline__ void prescale_one(float mn, float mx, float qmax, float &s, float &z) {
    const float range = mx - mn;
    s = range / qmax;
    if (!(s >= FLT_MIN)) s = 1.0f;                     // zero, subnormal or NaN scale
    z = __builtin_rintf((-mn) / s) + 0.0f;             // "+ 0" turns -0 into +0
}

// Min / max over the partials of channel c that the first pass of the reduction left in the
// workspace (granq_plan.h: channel_partials); the caller takes items start, start + stride, ...
__device__ inline void gather_channel(const float *__restrict__ ws_min, const float *__restrict__ ws_max,
                                      const ColPlan &plan, int64_t c, uint32_t start, uint32_t stride,
                                      float &mn, float &mx) {
    const ChannelPartials cp = channel_partials(plan, c);
    for (uint32_t i = start; i < cp.total; i += stride) {
        const int64_t at = channel_partial_slot(plan, c, cp, i);
        mn = __builtin_fminf(mn, ws_min[at]);
        mx = __builtin_fmaxf(mx, ws_max[at]);
    }
}

// Hand-over of a channel's parameters inside ONE launch (the forward that also finishes the
// reduction): scale in the low word, zero-point in the high word of a 64-bit slot per channel,
// written and read with single 64-bit accesses of device scope, so a reader sees either the
// marker or both parameters.  The marker is a NaN pattern that Eq. 5 never produces (a NaN
// scale becomes 1).
constexpr uint32_t kParamsPending = 0xFFFFFFFFu;

__device__ inline uint64_t pack_params(float s, float z) {
    return (uint64_t)__float_as_uint(s) | ((uint64_t)__float_as_uint(z) << 32);
}
__device__ inline uint64_t load_params(const uint64_t *slot) {
    return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline void publish_params(uint64_t *slot, uint64_t v) {
    __hip_atomic_store(slot, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// What the forward needs to finish the reduction itself (granq_calibrate_fakequant_fwd).
struct FinishArgs {
    const float *ws_min, *ws_max;    // partials of the first pass
    uint64_t *params;                // hand-over slots, one per channel; the first pass marked them pending
    float *ch_min, *ch_max, *scale, *zero_point;   // the caller's four vectors
    ColPlan rplan;                   // plan of the first pass (layout of the partials)
    int32_t finisher_rows;           // leading rows of the grid whose blocks finish one channel each
    int32_t spin_limit;              // polls before a waiting wavefront computes the parameters itself
};

// ---------------------------------------------------------------------------
// fake-quant forward and straight-through backward, column kernels
// ---------------------------------------------------------------------------

template <int MODE, int NS>
__device__ inline ChanRegs pick_chan(const ChanRegs (&c)[NS], int e, uint32_t split) {
    if (MODE == kOne) return c[0];
    if (MODE == kEach) return c[e < NS ? e : 0];
    ChanRegs r;
    const bool first = (uint32_t)e < split;
    r.s = first ? c[0].s : c[NS > 1 ? 1 : 0].s;
    r.z = first ? c[0].z : c[NS > 1 ? 1 : 0].z;
    r.r = first ? c[0].r : c[NS > 1 ? 1 : 0].r;
    return r;
}

// Shared prologue, first half: this lane's vectors within a row and the channels of their
// element groups.  GLUED: the plan may have glued rows (column -> column within the true row
// first).
template <typename T, int V, int MODE, bool GLUED = true>
__device__ inline void lane_columns(const ColPlan &plan, uint32_t j,
                                    int32_t (&ch)[V][Slots<MODE, T::VEC>::N], uint32_t (&split)[V],
                                    uint32_t (&cv)[V], bool (&active)[V]) {
    constexpr int VEC = T::VEC;
    constexpr int NS = Slots<MODE, VEC>::N;
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const uint32_t col = j * (uint32_t)plan.span + (threadIdx.x + v * kEBlock) * VEC;
        active[v] = col < (uint32_t)plan.row_len;
        cv[v] = col / VEC;
        const uint32_t tcol = GLUED ? true_column(col, plan) : col;
        split[v] = vector_channels<MODE, VEC, NS>(active[v] ? tcol : 0u, plan, ch[v]);
    }
}

// Second half: the channels' registers from the scale and zero-point vectors.
// Returns true when every channel this lane touches admits the fast quotient.
template <typename T, int V, int MODE, bool GLUED = true>
__device__ inline bool lane_setup(const ColPlan &plan, uint32_t j, const float *__restrict__ scale,
                                  const float *__restrict__ zero_point,
                                  ChanRegs (&cr)[V][Slots<MODE, T::VEC>::N], uint32_t (&split)[V],
                                  uint32_t (&cv)[V], bool (&active)[V]) {
    constexpr int NS = Slots<MODE, T::VEC>::N;
    int32_t ch[V][NS];
    lane_columns<T, V, MODE, GLUED>(plan, j, ch, split, cv, active);
    bool fast = GRANQ_FAST_QUOTIENT != 0;
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int e = 0; e < NS; ++e) {
            const float s = scale[ch[v][e]], z = zero_point[ch[v][e]];
            cr[v][e].s = s;
            cr[v][e].z = z;
            cr[v][e].r = 1.0f / s;
            fast = fast && quotient_fast_ok(s, z);
        }
    return fast;
}

#ifndef GRANQ_MASK_NT
#define GRANQ_MASK_NT 0
#endif
__device__ inline void store_mask_byte(uint8_t *p, uint8_t v) {
#if GRANQ_MASK_NT
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// What the forward writes besides x_hat.
constexpr int kNoExtra = 0;   // nothing
constexpr int kCodes = 1;     // one byte per element: the clamped code q
constexpr int kMask = 2;      // one bit per element: 1 where the clamp was inactive (the
                              // straight-through gate), bit (i & 7) of byte (i >> 3), i the
                              // flat NCHW index
constexpr int kCodesOnly = 3; // the codes, and x_hat is not written at all
constexpr int kPacked = 4;    // codes of at most four bits, two per byte: element i in nibble (i & 1) of byte i >> 1
constexpr int kPackedOnly = 5;// those, and x_hat is not written at all

// Rows r .. r + nrows - 1 of this lane's vectors, all loads issued together.
template <typename T, int V, int U, bool NT>
__device__ inline void fwd_load(const typename T::vec_t *x, int64_t row_vecs, int64_t r, int nrows,
                                const uint32_t (&cv)[V], const bool (&active)[V],
                                typename T::vec_t (&in)[U][V]) {
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int v = 0; v < V; ++v)
            if (u < nrows && active[v]) in[u][v] = load_vec<NT>(x + (r + u) * row_vecs + cv[v]);
}

// Quantize, clamp, dequantize and store what fwd_load fetched.
template <typename T, int V, int U, int MODE, int EXTRA, bool FAST>
__device__ inline void fwd_finish_rows(const typename T::vec_t (&in)[U][V], typename T::vec_t *x_hat,
                                       void *__restrict__ extra, float qmax, int64_t row_vecs, int64_t r,
                                       int nrows, const ChanRegs (&cr)[V][Slots<MODE, T::VEC>::N],
                                       const uint32_t (&split)[V], const uint32_t (&cv)[V],
                                       const bool (&active)[V]) {
    constexpr int VEC = T::VEC;
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int v = 0; v < V; ++v) {
            uint32_t gate_bits = 0;                    // bit e: element e passes the gate
            if (u < nrows && active[v]) {
                float f[VEC], q[VEC];
                T::unpack(in[u][v], f);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const ChanRegs c = pick_chan<MODE>(cr[v], e, split[v]);
                    const float code = code_of<FAST>(f[e], c);
                    q[e] = clamp_code(code, qmax);
                    // the clamp left the code alone <=> 0 <= code <= qmax (-0 == +0; NaN fails)
                    if (EXTRA == kMask) gate_bits |= (code == q[e] ? 1u : 0u) << e;
                    if (EXTRA != kCodesOnly && EXTRA != kPackedOnly) f[e] = dequant(q[e], c.s, c.z);
                }
                const int64_t at = (r + u) * row_vecs + cv[v];
                if (EXTRA != kCodesOnly && EXTRA != kPackedOnly) store_vec(x_hat + at, T::pack(f));
                if (EXTRA == kCodes || EXTRA == kCodesOnly)
                    store_vec((typename T::code_t *)extra + at, T::pack_codes(q));
                if (EXTRA == kPacked || EXTRA == kPackedOnly)
                    store_vec((typename T::code4_t *)extra + at, T::pack_codes4(q));
            }
            if (EXTRA == kMask && u < nrows) {         // wave-uniform condition: all lanes take part
                // byte index of this lane's vector; VEC == 8: one byte per lane, VEC == 4: two
                // neighbouring lanes share a byte (the row length is a multiple of 8 on this path,
                // so a pair is active or inactive together and starts on a byte boundary)
                const int64_t byte_at = ((r + u) * row_vecs + cv[v]) * VEC / 8;
                uint8_t *mask = (uint8_t *)extra;
                if (VEC == 8) {
                    if (active[v]) store_mask_byte(mask + byte_at, (uint8_t)gate_bits);
                } else {
                    const uint32_t other = (uint32_t)__builtin_amdgcn_update_dpp(
                        0, (int)gate_bits, kDppQuadSwap1, 0xF, 0xF, false);   // lane ^ 1
                    if (active[v] && (threadIdx.x & 1u) == 0) store_mask_byte(mask + byte_at, (uint8_t)(gate_bits | (other << 4)));
                }
            }
        }
}

template <typename T, int V, int U, int MODE, int EXTRA, bool FAST, bool NT>
__device__ inline void fwd_rows(const typename T::vec_t *x,
                                typename T::vec_t *x_hat, void *__restrict__ extra,
                                float qmax, int64_t row_vecs, int64_t r, int nrows,
                                const ChanRegs (&cr)[V][Slots<MODE, T::VEC>::N],
                                const uint32_t (&split)[V], const uint32_t (&cv)[V],
                                const bool (&active)[V]) {
    typename T::vec_t in[U][V];
    fwd_load<T, V, U, NT>(x, row_vecs, r, nrows, cv, active, in);
    fwd_finish_rows<T, V, U, MODE, EXTRA, FAST>(in, x_hat, extra, qmax, row_vecs, r, nrows, cr, split, cv, active);
}

template <typename T, int V, int U, int MODE, int EXTRA>
__global__ __launch_bounds__(kEBlock) void fq_fwd_cols(
    const typename T::vec_t *x, typename T::vec_t *x_hat,
    void *__restrict__ extra, const float *__restrict__ scale,
    const float *__restrict__ zero_point, float qmax, ColPlan plan)
{
    constexpr int NS = Slots<MODE, T::VEC>::N;
    const uint32_t j = GRANQ_FWD_REVERSE ? gridDim.x - 1 - blockIdx.x : blockIdx.x;
    const uint32_t p = GRANQ_FWD_REVERSE ? gridDim.y - 1 - blockIdx.y : blockIdx.y;
    const int64_t row_vecs = plan.row_len / T::VEC;

    ChanRegs cr[V][NS];
    uint32_t split[V], cv[V];
    bool active[V];
    // wave-uniform: if any lane's channel needs the general division, the whole wavefront takes it
    const bool fast = __all(lane_setup<T, V, MODE>(plan, j, scale, zero_point, cr, split, cv, active));

    const int64_t r0 = (int64_t)p * plan.rows_per_group;
    const int64_t r1 = (r0 + plan.rows_per_group < plan.rows) ? r0 + plan.rows_per_group : plan.rows;
    int64_t r = r0;
    const bool nt = r0 < plan.nt_row_end;              // block-uniform
    if (!fast) {
        for (; r < r1; ++r)
            fwd_rows<T, V, 1, MODE, EXTRA, false, false>(x, x_hat, extra, qmax, row_vecs, r, 1, cr, split, cv, active);
    } else if (nt) {
        for (; r + U <= r1; r += U)
            fwd_rows<T, V, U, MODE, EXTRA, true, true>(x, x_hat, extra, qmax, row_vecs, r, U, cr, split, cv, active);
        if (r < r1)
            fwd_rows<T, V, U, MODE, EXTRA, true, true>(x, x_hat, extra, qmax, row_vecs, r, (int)(r1 - r), cr, split, cv, active);
    } else {
        for (; r + U <= r1; r += U)
            fwd_rows<T, V, U, MODE, EXTRA, true, false>(x, x_hat, extra, qmax, row_vecs, r, U, cr, split, cv, active);
        if (r < r1)
            fwd_rows<T, V, U, MODE, EXTRA, true, false>(x, x_hat, extra, qmax, row_vecs, r, (int)(r1 - r), cr, split, cv, active);
    }
}

// Prologue of the forward that finishes the reduction: as lane_setup, but the parameters come
// from the hand-over slots, which the finisher blocks of the same launch fill.
// params_poll: one look at the slots of this lane's channels; true if any is still pending.
template <int V, int NS>
__device__ inline bool params_poll(const FinishArgs &fa, const int32_t (&ch)[V][NS], uint64_t (&pk)[V][NS],
                                   bool first) {
    bool pending = false;
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int e = 0; e < NS; ++e)
            if (first || (uint32_t)pk[v][e] == kParamsPending) {
                pk[v][e] = load_params(fa.params + ch[v][e]);
                pending = pending || (uint32_t)pk[v][e] == kParamsPending;
            }
    return pending;
}

// params_wait: a wavefront that found a slot pending polls it; after spin_limit polls it stops
// waiting and derives the parameters from the partials itself (the same operations in the
// same order, hence the same bits), so no wavefront ever depends on another one being
// scheduled.  Called by whole wavefronts.
template <int V, int NS>
__device__ inline void params_wait(const FinishArgs &fa, float qmax, const int32_t (&ch)[V][NS],
                                   uint64_t (&pk)[V][NS]) {
    bool pending = true;
    for (int32_t spins = 0; spins < fa.spin_limit && __any(pending); ++spins) {
        __builtin_amdgcn_s_sleep(4);
        pending = params_poll<V, NS>(fa, ch, pk, false);
    }
    if (!__any(pending)) return;
    const uint32_t lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int e = 0; e < NS; ++e) {
            bool mine = (uint32_t)pk[v][e] == kParamsPending;
            uint64_t waiting;
            while ((waiting = __ballot(mine)) != 0) {
                // one pending channel at a time, all 64 lanes on its partials
                const int leader = __builtin_ctzll(waiting);
                const int32_t c = __builtin_amdgcn_readlane(ch[v][e], leader);
                float mn = __builtin_inff(), mx = -__builtin_inff();
                gather_channel(fa.ws_min, fa.ws_max, fa.rplan, c, lane, kWave, mn, mx);
                mn = wave_min(mn);
                mx = wave_max(mx);
                float s, z;
                prescale_one(mn, mx, qmax, s, z);
                if (mine && ch[v][e] == c) {
                    pk[v][e] = pack_params(s, z);
                    mine = false;
                }
            }
        }
}

template <int V, int NS>
__device__ inline bool params_unpack(const uint64_t (&pk)[V][NS], ChanRegs (&cr)[V][NS]) {
    bool fast = GRANQ_FAST_QUOTIENT != 0;
#pragma unroll
    for (int v = 0; v < V; ++v)
#pragma unroll
        for (int e = 0; e < NS; ++e) {
            const float s = __uint_as_float((uint32_t)pk[v][e]);
            const float z = __uint_as_float((uint32_t)(pk[v][e] >> 32));
            cr[v][e].s = s;
            cr[v][e].z = z;
            cr[v][e].r = 1.0f / s;
            fast = fast && quotient_fast_ok(s, z);
        }
    return fast;
}

// granq_calibrate_fakequant_fwd's second launch: the forward, and in its leading
// `finisher_rows` rows of blocks the end of the reduction.  A finisher wavefront owns one
// channel: it gathers the channel's partials, applies Eq. 5, writes the caller's four
// vectors and publishes scale and zero-point in the channel's hand-over slot.  The other
// blocks are fq_fwd_cols with the prologue above.  Finishers have the lowest block indices,
// so they are dispatched first; nothing depends on that beyond speed.
template <typename T, int V, int U, int MODE, int EXTRA>
__global__ __launch_bounds__(kEBlock) void fq_fwd_finish_cols(
    const typename T::vec_t *x, typename T::vec_t *x_hat,
    void *__restrict__ extra, float qmax, ColPlan plan, FinishArgs fa)
{
    constexpr int NS = Slots<MODE, T::VEC>::N;
    if ((int32_t)blockIdx.y < fa.finisher_rows) {
        const int64_t c = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * (kEBlock / kWave) + threadIdx.x / kWave;
        if (c >= fa.rplan.channels) return;            // wave-uniform
        float mn = __builtin_inff(), mx = -__builtin_inff();
        gather_channel(fa.ws_min, fa.ws_max, fa.rplan, c, threadIdx.x & (kWave - 1), kWave, mn, mx);
        mn = wave_min(mn);
        mx = wave_max(mx);
        if ((threadIdx.x & (kWave - 1)) == 0) {
            float s, z;
            prescale_one(mn, mx, qmax, s, z);
            publish_params(fa.params + c, pack_params(s, z));
            fa.ch_min[c] = mn;
            fa.ch_max[c] = mx;
            fa.scale[c] = s;
            fa.zero_point[c] = z;
        }
        return;
    }
    const uint32_t rows_of_grid = gridDim.y - (uint32_t)fa.finisher_rows;
    const uint32_t by = blockIdx.y - (uint32_t)fa.finisher_rows;
    const uint32_t j = GRANQ_FWD_REVERSE ? gridDim.x - 1 - blockIdx.x : blockIdx.x;
    const uint32_t p = GRANQ_FWD_REVERSE ? rows_of_grid - 1 - by : by;
    const int64_t row_vecs = plan.row_len / T::VEC;
    const int64_t r0 = (int64_t)p * plan.rows_per_group;
    const int64_t r1 = (r0 + plan.rows_per_group < plan.rows) ? r0 + plan.rows_per_group : plan.rows;
    const bool nt = r0 < plan.nt_row_end;              // block-uniform

    int32_t ch[V][NS];
    ChanRegs cr[V][NS];
    uint32_t split[V], cv[V];
    bool active[V];
    uint64_t pk[V][NS];
    lane_columns<T, V, MODE, true>(plan, j, ch, split, cv, active);
    int64_t r = r0;
    // The blocks that start before the finishers are through (the first wave of the launch) find
    // their parameters pending: they fetch their first rows before they wait, so that the
    // finishers' latency hides behind the loads.  Every later block takes the ordinary order,
    // parameters first (that order streams faster).
    typename T::vec_t first_rows[U][V];
    int first_n = 0;
    if (__any(params_poll<V, NS>(fa, ch, pk, true))) { // wave-uniform
        first_n = (int)(r1 - r0 < U ? r1 - r0 : U);
        if (nt) fwd_load<T, V, U, true>(x, row_vecs, r0, first_n, cv, active, first_rows);
        else fwd_load<T, V, U, false>(x, row_vecs, r0, first_n, cv, active, first_rows);
        params_wait<V, NS>(fa, qmax, ch, pk);
    }
    // wave-uniform: if any lane's channel needs the general division, the whole wavefront takes it
    const bool fast = __all(params_unpack<V, NS>(pk, cr));
    if (first_n > 0) {
        if (fast) fwd_finish_rows<T, V, U, MODE, EXTRA, true>(first_rows, x_hat, extra, qmax, row_vecs, r0, first_n, cr, split, cv, active);
        else fwd_finish_rows<T, V, U, MODE, EXTRA, false>(first_rows, x_hat, extra, qmax, row_vecs, r0, first_n, cr, split, cv, active);
        r = r0 + first_n;
    }
    if (!fast) {
        for (; r < r1; ++r)
            fwd_rows<T, V, 1, MODE, EXTRA, false, false>(x, x_hat, extra, qmax, row_vecs, r, 1, cr, split, cv, active);
    } else if (nt) {
        for (; r + U <= r1; r += U)
            fwd_rows<T, V, U, MODE, EXTRA, true, true>(x, x_hat, extra, qmax, row_vecs, r, U, cr, split, cv, active);
        if (r < r1)
            fwd_rows<T, V, U, MODE, EXTRA, true, true>(x, x_hat, extra, qmax, row_vecs, r, (int)(r1 - r), cr, split, cv, active);
    } else {
        for (; r + U <= r1; r += U)
            fwd_rows<T, V, U, MODE, EXTRA, true, false>(x, x_hat, extra, qmax, row_vecs, r, U, cr, split, cv, active);
        if (r < r1)
            fwd_rows<T, V, U, MODE, EXTRA, true, false>(x, x_hat, extra, qmax, row_vecs, r, (int)(r1 - r), cr, split, cv, active);
    }
}

template <typename T, int V, int U, int MODE, bool FAST, bool NT>
__device__ inline void bwd_rows(const typename T::vec_t *x,
                                const typename T::vec_t *dy,
                                typename T::vec_t *dx, float qmax, int64_t row_vecs,
                                int64_t r, int nrows, const ChanRegs (&cr)[V][Slots<MODE, T::VEC>::N],
                                const uint32_t (&split)[V], const uint32_t (&cv)[V],
                                const bool (&active)[V]) {
    constexpr int VEC = T::VEC;
    typename T::vec_t in[U][V], g[U][V];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int v = 0; v < V; ++v)
            if (u < nrows && active[v]) {
                const int64_t at = (r + u) * row_vecs + cv[v];
                in[u][v] = load_vec<NT>(x + at);
                g[u][v] = load_vec<NT>(dy + at);
            }
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int v = 0; v < V; ++v)
            if (u < nrows && active[v]) {
                float f[VEC];
                bool keep[VEC];
                T::unpack(in[u][v], f);
#pragma unroll
                for (int e = 0; e < VEC; ++e)
                    keep[e] = in_range(code_of<FAST>(f[e], pick_chan<MODE>(cr[v], e, split[v])), qmax);
                store_vec(dx + (r + u) * row_vecs + cv[v], T::gate(g[u][v], keep));
            }
}

// GLUED is a template argument here because a block of the backward is a single row of one
// vector per lane: what its prologue loads and tests shows in the kernel's time (0.4 % measured).
template <typename T, int V, int U, bool GLUED, int MODE>
__global__ __launch_bounds__(kEBlock) void fq_bwd_cols(
    const typename T::vec_t *x, const typename T::vec_t *dy,
    typename T::vec_t *dx, const float *__restrict__ scale,
    const float *__restrict__ zero_point, float qmax, ColPlan plan)
{
    constexpr int NS = Slots<MODE, T::VEC>::N;
    const uint32_t j = blockIdx.x;
    const uint32_t p = blockIdx.y;
    const int64_t row_vecs = plan.row_len / T::VEC;

    ChanRegs cr[V][NS];
    uint32_t split[V], cv[V];
    bool active[V];
    // wave-uniform: if any lane's channel needs the general division, the whole wavefront takes it
    const bool fast = __all(lane_setup<T, V, MODE, GLUED>(plan, j, scale, zero_point, cr, split, cv, active));

    const int64_t r0 = (int64_t)p * plan.rows_per_group;
    const int64_t r1 = (r0 + plan.rows_per_group < plan.rows) ? r0 + plan.rows_per_group : plan.rows;
    int64_t r = r0;
    const bool nt = r0 < plan.nt_row_end;              // block-uniform
    if (!fast) {
        for (; r < r1; ++r)
            bwd_rows<T, V, 1, MODE, false, false>(x, dy, dx, qmax, row_vecs, r, 1, cr, split, cv, active);
    } else if (nt) {
        for (; r + U <= r1; r += U)
            bwd_rows<T, V, U, MODE, true, true>(x, dy, dx, qmax, row_vecs, r, U, cr, split, cv, active);
        if (r < r1)
            bwd_rows<T, V, U, MODE, true, true>(x, dy, dx, qmax, row_vecs, r, (int)(r1 - r), cr, split, cv, active);
    } else {
        for (; r + U <= r1; r += U)
            bwd_rows<T, V, U, MODE, true, false>(x, dy, dx, qmax, row_vecs, r, U, cr, split, cv, active);
        if (r < r1)
            bwd_rows<T, V, U, MODE, true, false>(x, dy, dx, qmax, row_vecs, r, (int)(r1 - r), cr, split, cv, active);
    }
}

// Backward from the forward's gate bits: dx = dy where the bit is set, else 0.
// Reads dy and one bit per element instead of x and dy.
template <typename T, int U, bool NT>
__global__ __launch_bounds__(kEBlock) void fq_bwd_mask_cols(
    const typename T::vec_t *dy, const uint8_t *__restrict__ mask,
    typename T::vec_t *dx, ColPlan plan)
{
    constexpr int VEC = T::VEC;
    const int64_t row_vecs = plan.row_len / VEC;
    const uint32_t col = blockIdx.x * (uint32_t)plan.span + threadIdx.x * VEC;
    if (col >= (uint32_t)plan.row_len) return;
    const uint32_t cv = col / VEC;
    const int64_t r0 = (int64_t)blockIdx.y * plan.rows_per_group;
    const int64_t r1 = (r0 + plan.rows_per_group < plan.rows) ? r0 + plan.rows_per_group : plan.rows;
    for (int64_t r = r0; r < r1; r += U) {
        typename T::vec_t g[U];
        uint32_t bits[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (r + u < r1) {
                const int64_t at = (r + u) * row_vecs + cv;
                g[u] = load_vec<NT>(dy + at);
                bits[u] = mask[at * VEC / 8];
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (r + u < r1) {
                const uint32_t b = VEC == 8 ? bits[u] : (bits[u] >> (4 * (threadIdx.x & 1u)));
                bool keep[VEC];
#pragma unroll
                for (int e = 0; e < VEC; ++e) keep[e] = (b >> e) & 1u;
                store_vec(dx + (r + u) * row_vecs + cv, T::gate(g[u], keep));
            }
    }
}

// Any shape: one thread per mask byte (eight consecutive elements).
template <typename T>
__global__ __launch_bounds__(kBlock) void mask_from_x_bytes(
    const void *__restrict__ x, const float *__restrict__ scale, const float *__restrict__ zero_point,
    float qmax, int64_t c, int64_t hw, int64_t total, uint8_t *__restrict__ mask)
{
    const int64_t nbytes = (total + 7) / 8;
    for (int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x; b < nbytes; b += (int64_t)gridDim.x * kBlock) {
        uint32_t bits = 0;
        for (int k = 0; k < 8; ++k) {
            const int64_t i = b * 8 + k;
            if (i < total) {
                const int64_t ic = (i / hw) % c;
                const float u = raw_code(T::load1(x, i), scale[ic], zero_point[ic]);
                bits |= (in_range(u, qmax) ? 1u : 0u) << k;
            }
        }
        mask[b] = (uint8_t)bits;
    }
}

// Any shape: one thread per packed byte (two consecutive elements): codes two per byte, and
// x_hat where asked for (it may alias x: a thread reads its elements before it writes them).
template <typename T>
__global__ __launch_bounds__(kBlock) void fwd_packed_bytes(
    const void *x, void *x_hat, const float *__restrict__ scale, const float *__restrict__ zero_point,
    float qmax, int64_t c, int64_t hw, int64_t total, uint8_t *__restrict__ packed)
{
    const int64_t nbytes = (total + 1) / 2;
    for (int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x; b < nbytes; b += (int64_t)gridDim.x * kBlock) {
        float xv[2], sv[2], zv[2];
        uint32_t byte = 0;
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int64_t i = b * 2 + k;
            if (i < total) {
                const int64_t ic = (i / hw) % c;
                xv[k] = T::load1(x, i);
                sv[k] = scale[ic];
                zv[k] = zero_point[ic];
            }
        }
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int64_t i = b * 2 + k;
            if (i < total) {
                const float q = clamp_code(raw_code(xv[k], sv[k], zv[k]), qmax);
                byte |= (uint32_t)q << (4 * k);
                if (x_hat) T::store1(x_hat, i, dequant(q, sv[k], zv[k]));
            }
        }
        packed[b] = (uint8_t)byte;
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void bwd_mask_bytes(
    const void *dy, const uint8_t *__restrict__ mask, int64_t total, void *dx)
{
    const int64_t nbytes = (total + 7) / 8;
    for (int64_t b = (int64_t)blockIdx.x * kBlock + threadIdx.x; b < nbytes; b += (int64_t)gridDim.x * kBlock) {
        const uint32_t bits = mask[b];
        for (int k = 0; k < 8; ++k) {
            const int64_t i = b * 8 + k;
            if (i < total) T::store_gated1(dx, dy, i, (bits >> k) & 1u);
        }
    }
}

// ---------------------------------------------------------------------------
// range reduce, column kernel (pass 1) and its pass 2
// ---------------------------------------------------------------------------
//
// Pass 1: every lane keeps a running min / max per element position of its
// vectors while walking down its rows.  At the end of the block the lanes'
// results are combined per channel: a wavefront whose lanes all hold the same
// channel reduces with DPP and issues one LDS atomic, otherwise each lane issues
// its own; the per-channel LDS slots are then written to the workspace as
// partials  ws[(p * J + j) * kmax + (channel - first channel of tile j)].
// Pass 2: one wavefront per channel gathers the partials of all column tiles
// that overlap the channel and of all row groups.

// End of a block's sweep: the lanes' running minima and maxima (one pair per element position of
// each of their V vectors, or one per vector in mode kOne) are combined per channel in LDS:
// keys[k] / keys[kmax + k] for channel (first channel of tile j) + k, as order-preserving
// integer keys.  A wavefront whose lanes all hold the same channel reduces with DPP and issues
// one LDS atomic, otherwise each lane issues its own.  The keys must have been initialised and a
// barrier passed; the caller places the barrier that follows.
template <typename T, int V, int MODE>
__device__ inline void lanes_to_channel_keys(const ColPlan &plan, uint32_t j, float (&mn)[V][MODE == kOne ? 1 : T::VEC],
                                             float (&mx)[V][MODE == kOne ? 1 : T::VEC], const uint32_t (&cv)[V],
                                             const bool (&active)[V], uint32_t *lds_keys) {
    constexpr int VEC = T::VEC;
    constexpr int NS = MODE == kOne ? 1 : VEC;
    const int32_t kmax = plan.kmax;
    const int32_t ch_first = (int32_t)fastdiv(j * (uint32_t)plan.span, plan.hw_div);
    constexpr int NG = Slots<MODE, VEC>::N;             // channel groups per vector
    // glued rows whose length divides the distance between a lane's vectors: all V vectors
    // belong to the same channels, so they are combined in registers and only the first one
    // goes to LDS (inactive vectors hold the identities)
    if (V > 1 && plan.v_same) {
#pragma unroll
        for (int v = 1; v < V; ++v)
#pragma unroll
            for (int e = 0; e < NS; ++e) {
                mn[0][e] = __builtin_fminf(mn[0][e], mn[v][e]);
                mx[0][e] = __builtin_fmaxf(mx[0][e], mx[v][e]);
            }
    }
#pragma unroll
    for (int v = 0; v < V; ++v) {
        if (v > 0 && plan.v_same) break;               // block-uniform
        // inactive lanes hold the identities and point at the tile's first channel; with glued
        // rows the channel follows from the column within the true row
        const uint32_t col = true_column(active[v] ? cv[v] * VEC : j * (uint32_t)plan.span, plan);
        int32_t ch[NG];
        const uint32_t split = vector_channels<MODE, VEC, NG>(col, plan, ch);
        float gmn[NG], gmx[NG];
        if (MODE == kTwo) {
            // fold the element positions into the (at most) two channels of the vector
            gmn[0] = gmn[NG - 1] = __builtin_inff();
            gmx[0] = gmx[NG - 1] = -__builtin_inff();
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const bool first = (uint32_t)e < split;
                const float a = mn[v][e < NS ? e : 0], b = mx[v][e < NS ? e : 0];
                gmn[0] = __builtin_fminf(gmn[0], first ? a : __builtin_inff());
                gmx[0] = __builtin_fmaxf(gmx[0], first ? b : -__builtin_inff());
                gmn[NG - 1] = __builtin_fminf(gmn[NG - 1], first ? __builtin_inff() : a);
                gmx[NG - 1] = __builtin_fmaxf(gmx[NG - 1], first ? -__builtin_inff() : b);
            }
        } else {
#pragma unroll
            for (int e = 0; e < NG; ++e) {
                gmn[e] = mn[v][e < NS ? e : 0];
                gmx[e] = mx[v][e < NS ? e : 0];
            }
        }
#pragma unroll
        for (int e = 0; e < NG; ++e) {
            const int32_t k = ch[e] - ch_first;
            const int32_t k_lead = __builtin_amdgcn_readfirstlane(k);
            if (__all(k == k_lead)) {
                float wmn = wave_min(gmn[e]);
                float wmx = wave_max(gmx[e]);
                if ((threadIdx.x & (kWave - 1)) == 0) {
                    atomicMin(&lds_keys[k_lead], float_key(wmn));
                    atomicMax(&lds_keys[kmax + k_lead], float_key(wmx));
                }
            } else {
                atomicMin(&lds_keys[k], float_key(gmn[e]));
                atomicMax(&lds_keys[kmax + k], float_key(gmx[e]));
            }
        }
    }

}

// What the first pass does besides writing partials.
struct Pass1Extra {
    uint64_t *params;        // non-null: mark every channel's hand-over slot pending for the
                             // forward that finishes the reduction (row group 0 does it)
    int32_t direct;          // > 0: there is one row group and every channel lies inside one column
                             // tile, which holds `direct` channels: the block's results are final and
                             // go straight to the vectors below (no partials, no second pass)
    float *ch_min, *ch_max;
    float *scale, *zero_point;   // null: ranges only
    float qmax;
};

template <typename T, int V, int MODE>
__global__ __launch_bounds__(kRBlock) void range_cols_pass1(
    const typename T::vec_t *__restrict__ x, float *__restrict__ ws_min,
    float *__restrict__ ws_max, ColPlan plan, Pass1Extra px)
{
    constexpr int VEC = T::VEC;
    constexpr int NS = MODE == kOne ? 1 : VEC;           // running min/max per element position
    constexpr int U = GRANQ_R_UNROLL;
    using vec_t = typename T::vec_t;
    extern __shared__ uint32_t lds_keys[];          // [kmax] min keys, then [kmax] max keys

    const uint32_t j = blockIdx.x;
    const uint32_t p = blockIdx.y;
    const int64_t row_vecs = plan.row_len / VEC;
    const int32_t kmax = plan.kmax;

    for (int i = threadIdx.x; i < kmax; i += kRBlock) {
        lds_keys[i] = kKeyPosInf;
        lds_keys[kmax + i] = kKeyNegInf;
    }

    float mn[V][NS], mx[V][NS];
    uint32_t cv[V];
    bool active[V];
#pragma unroll
    for (int v = 0; v < V; ++v) {
        const uint32_t col = j * (uint32_t)plan.span + (threadIdx.x + v * kRBlock) * VEC;
        active[v] = col < (uint32_t)plan.row_len;
        cv[v] = col / VEC;
#pragma unroll
        for (int e = 0; e < NS; ++e) {
            mn[v][e] = __builtin_inff();
            mx[v][e] = -__builtin_inff();
        }
    }

    const int64_t r0 = (int64_t)p * plan.rows_per_group;
    const int64_t r1 = (r0 + plan.rows_per_group < plan.rows) ? r0 + plan.rows_per_group : plan.rows;

    auto body = [&](int64_t r, const int nrows, auto nt_tag) {
        constexpr bool NT = decltype(nt_tag)::value;
        vec_t in[U][V];
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int v = 0; v < V; ++v)
                if (u < nrows && active[v]) in[u][v] = load_vec<NT>(x + (r + u) * row_vecs + cv[v]);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int v = 0; v < V; ++v)
                if (u < nrows && active[v]) {
                    float f[VEC];
                    T::unpack(in[u][v], f);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        mn[v][MODE == kOne ? 0 : e] = __builtin_fminf(mn[v][MODE == kOne ? 0 : e], f[e]);
                        mx[v][MODE == kOne ? 0 : e] = __builtin_fmaxf(mx[v][MODE == kOne ? 0 : e], f[e]);
                    }
                }
    };

    int64_t r = r0;
    if (r0 < plan.nt_row_end) {                        // block-uniform
        for (; r + U <= r1; r += U) body(r, U, std::true_type{});
        if (r < r1) body(r, (int)(r1 - r), std::true_type{});
    } else {
        for (; r + U <= r1; r += U) body(r, U, std::false_type{});
        if (r < r1) body(r, (int)(r1 - r), std::false_type{});
    }

    __syncthreads();                                   // LDS slots initialised

    lanes_to_channel_keys<T, V, MODE>(plan, j, mn, mx, cv, active, lds_keys);
    const int32_t ch_first = (int32_t)fastdiv(j * (uint32_t)plan.span, plan.hw_div);

    __syncthreads();

    if (px.direct > 0) {
        for (int i = threadIdx.x; i < px.direct; i += kRBlock) {
            const int32_t c = ch_first + i;
            if (c >= plan.channels) break;
            const float mn = key_float(lds_keys[i]), mx = key_float(lds_keys[kmax + i]);
            px.ch_min[c] = mn;
            px.ch_max[c] = mx;
            if (px.scale) {
                float sc, zp;
                prescale_one(mn, mx, px.qmax, sc, zp);
                px.scale[c] = sc;
                px.zero_point[c] = zp;
            }
        }
        return;
    }
    const int64_t slot = partial_slot(plan, p, j, 0);
    for (int i = threadIdx.x; i < kmax; i += kRBlock) {
        ws_min[slot + i] = key_float(lds_keys[i]);
        ws_max[slot + i] = key_float(lds_keys[kmax + i]);
        if (px.params && p == 0 && ch_first + i < plan.channels) px.params[ch_first + i] = kParamsPending;
    }
}

// `scale` / `zero_point` may be null (ranges only); otherwise Eq. 5 is applied
// to the channel's range in the same launch.  WPC wavefronts share one channel:
// 1 where a channel has a few hundred partials at most, 4 (the whole block, combined
// through LDS) where it has thousands (glued rows: one partial per row group).
template <int WPC>
__global__ __launch_bounds__(kBlock) void range_cols_pass2(
    const float *__restrict__ ws_min, const float *__restrict__ ws_max,
    float *__restrict__ ch_min, float *__restrict__ ch_max, ColPlan plan,
    float qmax, float *__restrict__ scale, float *__restrict__ zero_point)
{
    constexpr int kPerBlock = kBlock / kWave / WPC;    // channels per block
    __shared__ float part[2][kBlock / kWave];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t c = (int64_t)blockIdx.x * kPerBlock + wave / WPC;
    const bool live = c < plan.channels;               // wave-uniform
    float mn = __builtin_inff(), mx = -__builtin_inff();
    if (live) {
        gather_channel(ws_min, ws_max, plan, c, (uint32_t)((wave % WPC) * kWave + lane), kWave * WPC, mn, mx);
        mn = wave_min(mn);
        mx = wave_max(mx);
    }
    if (WPC > 1) {
        if (lane == 0) {
            part[0][wave] = mn;
            part[1][wave] = mx;
        }
        __syncthreads();
        if (wave % WPC == 0) {
#pragma unroll
            for (int w = 1; w < WPC; ++w) {
                mn = __builtin_fminf(mn, part[0][wave + w]);
                mx = __builtin_fmaxf(mx, part[1][wave + w]);
            }
        }
    }
    if (live && lane == 0 && wave % WPC == 0) {
        ch_min[c] = mn;
        ch_max[c] = mx;
        if (scale) {
            float sc, zp;
            prescale_one(mn, mx, qmax, sc, zp);
            scale[c] = sc;
            zero_point[c] = zp;
        }
    }
}

// ---------------------------------------------------------------------------
// ranges, parameters and forward in ONE launch, the tensor resident in registers
// ---------------------------------------------------------------------------
//
// Every block loads its slice (a column tile x up to R rows, one 16-byte vector per lane and
// row) once and keeps it in registers.  It reduces the slice to per-channel partial minima
// and maxima, publishes them, and counts itself in at the channels its tile overlaps (one
// 64-bit arrival counter per channel, never reset: arrival number a of a call belongs to
// epoch a / expected).  The block that arrives last at a channel gathers the channel's
// partials, applies Eq. 5, writes the caller's four vectors and publishes scale and
// zero-point in the channel's parameter slot, tagged with the epoch's parity in the sign bit of
// the (always positive) scale.  Every block then waits for the slots of its lanes' channels
// to carry this epoch's tag and quantizes what it holds.
//
// Data crosses blocks only through device-scope accesses: partials and slots are written and
// read with single atomic stores / loads that bypass the per-die L2, a block's partial stores
// are complete (s_waitcnt) before it counts itself in, and the last arriver reads the partials
// only after its own arrival returned.
//
// Nothing depends on all blocks being on the chip at once except speed: a wavefront that has
// polled spin_limit times stops waiting and computes its channels' ranges by scanning the
// channels itself (x is still intact: this form does not run in place).
struct ResidentArgs {
    const void *x;
    void *x_hat;                     // may be null (codes only)
    uint8_t *codes;                  // may be null
    float *ch_min, *ch_max, *scale, *zero_point;
    float *ws_min, *ws_max;          // partials
    unsigned long long *arrive;      // arrivals per channel since the state was zeroed
    uint64_t *params;                // scale (epoch tag in the sign bit) | zero-point << 32
    ColPlan plan;
    int64_t n, c, hw;                // the tensor's own dimensions (for the scan of a channel)
    float qmax;
    int32_t spin_limit;
};

__device__ inline void store_agent(float *p, float v) {
    __hip_atomic_store((uint32_t *)p, __float_as_uint(v), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float load_agent(const float *p) {
    return __uint_as_float(__hip_atomic_load((const uint32_t *)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// gather_channel with device-scope loads (the partials were written by blocks of this launch).
__device__ inline void gather_channel_agent(const float *ws_min, const float *ws_max, const ColPlan &plan,
                                            int64_t c, uint32_t start, uint32_t stride, float &mn, float &mx) {
    const ChannelPartials cp = channel_partials(plan, c);
    for (uint32_t i = start; i < cp.total; i += stride) {
        const int64_t at = channel_partial_slot(plan, c, cp, i);
        mn = __builtin_fminf(mn, load_agent(ws_min + at));
        mx = __builtin_fmaxf(mx, load_agent(ws_max + at));
    }
}

// Min / max of channel ch straight from the tensor, by one wavefront.
template <typename T>
__device__ inline void scan_channel(const void *x, int64_t n, int64_t c, int64_t hw, int64_t ch, float &mn, float &mx) {
    const int lane = threadIdx.x & (kWave - 1);
    mn = __builtin_inff();
    mx = -__builtin_inff();
    for (int64_t in = 0; in < n; ++in) {
        const int64_t base = (in * c + ch) * hw;
        for (int64_t k = lane; k < hw; k += kWave) {
            const float v = T::load1(x, base + k);
            mn = __builtin_fminf(mn, v);
            mx = __builtin_fmaxf(mx, v);
        }
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
}

template <typename T, int R, int MODE>
__global__ __launch_bounds__(kResBlock) void fq_resident_cols(ResidentArgs a)
{
    constexpr int VEC = T::VEC;
    constexpr int NR = MODE == kOne ? 1 : VEC;          // running min / max per element position
    constexpr int NS = Slots<MODE, VEC>::N;             // channel slots of a vector
    using vec_t = typename T::vec_t;
    extern __shared__ uint32_t lds_keys[];              // [kmax] min keys, then [kmax] max keys
    __shared__ uint32_t epoch_tag;
    const ColPlan &plan = a.plan;
    const uint32_t j = blockIdx.x, p = blockIdx.y;
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row_vecs = plan.row_len / VEC;
    const int32_t kmax = plan.kmax;
    for (int i = threadIdx.x; i < kmax; i += kResBlock) {
        lds_keys[i] = kKeyPosInf;
        lds_keys[kmax + i] = kKeyNegInf;
    }

    // 1. the slice, all loads in flight together
    const uint32_t col = j * (uint32_t)plan.span + threadIdx.x * VEC;
    const bool active1[1] = {col < (uint32_t)plan.row_len};
    const uint32_t cv1[1] = {col / VEC};
    const int64_t r0 = (int64_t)p * plan.rows_per_group;
    const int64_t r1 = (r0 + plan.rows_per_group < plan.rows) ? r0 + plan.rows_per_group : plan.rows;
    const int nrows = (int)(r1 - r0);                   // <= R
    vec_t in[R];
#pragma unroll
    for (int u = 0; u < R; ++u)
        if (u < nrows && active1[0]) in[u] = ((const vec_t *)a.x)[(r0 + u) * row_vecs + cv1[0]];
    float mn[1][NR], mx[1][NR];
#pragma unroll
    for (int e = 0; e < NR; ++e) {
        mn[0][e] = __builtin_inff();
        mx[0][e] = -__builtin_inff();
    }
#pragma unroll
    for (int u = 0; u < R; ++u)
        if (u < nrows && active1[0]) {
            float f[VEC];
            T::unpack(in[u], f);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                mn[0][MODE == kOne ? 0 : e] = __builtin_fminf(mn[0][MODE == kOne ? 0 : e], f[e]);
                mx[0][MODE == kOne ? 0 : e] = __builtin_fmaxf(mx[0][MODE == kOne ? 0 : e], f[e]);
            }
        }

    // 2. per-channel partials of the block
    __syncthreads();
    lanes_to_channel_keys<T, 1, MODE>(plan, j, mn, mx, cv1, active1, lds_keys);
    __syncthreads();

    // 3. publish, arrive, and finish the channels this block completes (first wavefront)
    const int32_t ch_first = (int32_t)fastdiv(j * (uint32_t)plan.span, plan.hw_div);
    if (threadIdx.x < kWave) {
        const uint32_t tile_end = (j + 1) * (uint32_t)plan.span < (uint32_t)plan.row_len ? (j + 1) * (uint32_t)plan.span
                                                                                         : (uint32_t)plan.row_len;
        int32_t ch_last = (int32_t)fastdiv(tile_end - 1, plan.hw_div);
        if (ch_last > plan.channels - 1) ch_last = plan.channels - 1;     // glued rows: one tile, all channels
        const int64_t slot = partial_slot(plan, p, j, 0);
        for (int i = lane; i < kmax; i += kWave) {
            store_agent(a.ws_min + slot + i, key_float(lds_keys[i]));
            store_agent(a.ws_max + slot + i, key_float(lds_keys[kmax + i]));
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");          // the partials have reached memory
        uint32_t tag = 0;
        for (int base = 0; base < kmax; base += kWave) {          // wave-uniform loop
            const int32_t c = ch_first + base + lane;
            const bool valid = c <= ch_last;
            unsigned long long old = 0;
            uint32_t expected = 1;
            if (valid) {
                expected = channel_partials(plan, c).total;
                old = __hip_atomic_fetch_add(a.arrive + c, 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            const unsigned long long epoch = old / expected;
            bool last = valid && (uint32_t)(old - epoch * expected) == expected - 1;
            if (base == 0) tag = (uint32_t)((epoch + 1) & 1u);    // lane 0 is valid; every channel is in the same epoch
            uint64_t todo;
            while ((todo = __ballot(last)) != 0) {                // one completed channel at a time
                const int leader = __builtin_ctzll(todo);
                const int32_t cl = __builtin_amdgcn_readlane(c, leader);
                float gmn = __builtin_inff(), gmx = -__builtin_inff();
                gather_channel_agent(a.ws_min, a.ws_max, plan, cl, lane, kWave, gmn, gmx);
                gmn = wave_min(gmn);
                gmx = wave_max(gmx);
                if (lane == leader) {
                    float sc, zp;
                    prescale_one(gmn, gmx, a.qmax, sc, zp);
                    const uint32_t my_tag = (uint32_t)((epoch + 1) & 1u);
                    publish_params(a.params + cl, (uint64_t)(__float_as_uint(sc) | (my_tag << 31)) |
                                                      ((uint64_t)__float_as_uint(zp) << 32));
                    a.ch_min[cl] = gmn;
                    a.ch_max[cl] = gmx;
                    a.scale[cl] = sc;
                    a.zero_point[cl] = zp;
                    last = false;
                }
            }
        }
        if (lane == 0) epoch_tag = __builtin_amdgcn_readfirstlane(tag);
    }
    __syncthreads();
    const uint32_t want = epoch_tag;

    // 4. wait for the parameters of this lane's channels
    int32_t ch[NS];
    const uint32_t split = vector_channels<MODE, VEC, NS>(active1[0] ? true_column(col, plan) : 0u, plan, ch);
    uint64_t pk[NS];
    auto poll = [&]() {
        bool pending = false;
#pragma unroll
        for (int e = 0; e < NS; ++e) {
            pk[e] = load_params(a.params + ch[e]);
            pending = pending || (((uint32_t)pk[e]) >> 31) != want;
        }
        return pending;
    };
    bool pending = poll();
    for (int32_t spins = 0; spins < a.spin_limit && __any(pending); ++spins) {
        __builtin_amdgcn_s_sleep(4);
        pending = poll();
    }
    if (__any(pending)) {                               // wave-uniform: scan the pending channels ourselves
#pragma unroll
        for (int e = 0; e < NS; ++e) {
            bool mine = (((uint32_t)pk[e]) >> 31) != want;
            uint64_t waiting;
            while ((waiting = __ballot(mine)) != 0) {
                const int leader = __builtin_ctzll(waiting);
                const int32_t cl = __builtin_amdgcn_readlane(ch[e], leader);
                float gmn, gmx, sc, zp;
                scan_channel<T>(a.x, a.n, a.c, a.hw, cl, gmn, gmx);
                prescale_one(gmn, gmx, a.qmax, sc, zp);
                if (mine && ch[e] == cl) {
                    pk[e] = pack_params(sc, zp) | ((uint64_t)want << 31);
                    mine = false;
                }
            }
        }
    }
    ChanRegs cr[NS];
    bool fast = GRANQ_FAST_QUOTIENT != 0;
#pragma unroll
    for (int e = 0; e < NS; ++e) {
        cr[e].s = __uint_as_float((uint32_t)pk[e] & 0x7FFFFFFFu);
        cr[e].z = __uint_as_float((uint32_t)(pk[e] >> 32));
        cr[e].r = 1.0f / cr[e].s;
        fast = fast && quotient_fast_ok(cr[e].s, cr[e].z);
    }
    fast = __all(fast);

    // 5. quantize, clamp, dequantize what the block holds
    auto finish = [&](auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll
        for (int u = 0; u < R; ++u)
            if (u < nrows && active1[0]) {
                float f[VEC], q[VEC];
                T::unpack(in[u], f);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const ChanRegs cc = pick_chan<MODE>(cr, e, split);
                    q[e] = clamp_code(code_of<FAST>(f[e], cc), a.qmax);
                    f[e] = dequant(q[e], cc.s, cc.z);
                }
                const int64_t at = (r0 + u) * row_vecs + cv1[0];
                if (a.x_hat) store_vec((vec_t *)a.x_hat + at, T::pack(f));
                if (a.codes) store_vec((typename T::code_t *)a.codes + at, T::pack_codes(q));
            }
    };
    if (fast) finish(std::true_type{});
    else finish(std::false_type{});
}

// ---------------------------------------------------------------------------
// element-wise fallbacks ("row" kernels): any shape, any element alignment
// ---------------------------------------------------------------------------

// Block (c, p, q): channel c, rows [p*rpg, (p+1)*rpg), piece q of every slab.  Per-lane
// min/max, DPP within the wavefront, LDS across the four wavefronts, one partial per block.
template <typename T>
__global__ __launch_bounds__(kBlock) void range_rows_pass1(
    const void *__restrict__ x, float *__restrict__ ws_min, float *__restrict__ ws_max,
    int64_t n, int64_t c, int64_t hw, RowPlan plan)
{
    __shared__ float part[2][kBlock / kWave];
    const int64_t ic = blockIdx.x % c;
    const int64_t pq = blockIdx.x / c;                 // (row group, piece), piece fastest
    const int64_t p = pq / plan.chunks, q = pq % plan.chunks;
    const int64_t r0 = p * plan.rows_per_group;
    const int64_t r1 = (r0 + plan.rows_per_group < n) ? r0 + plan.rows_per_group : n;
    const int64_t k0 = q * plan.chunk_len;
    const int64_t k1 = k0 + plan.chunk_len < hw ? k0 + plan.chunk_len : hw;
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (int64_t in = r0; in < r1; ++in) {
        const int64_t base = (in * c + ic) * hw;
        for (int64_t k = k0 + threadIdx.x; k < k1; k += kBlock) {
            float v = T::load1(x, base + k);
            mn = __builtin_fminf(mn, v);
            mx = __builtin_fmaxf(mx, v);
        }
    }
    mn = wave_min(mn);
    mx = wave_max(mx);
    const int wave = threadIdx.x / kWave;
    if ((threadIdx.x & (kWave - 1)) == 0) {
        part[0][wave] = mn;
        part[1][wave] = mx;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        for (int w = 1; w < kBlock / kWave; ++w) {
            mn = __builtin_fminf(mn, part[0][w]);
            mx = __builtin_fmaxf(mx, part[1][w]);
        }
        ws_min[pq * c + ic] = mn;
        ws_max[pq * c + ic] = mx;
    }
}

// `groups`: partials per channel (row groups x pieces).
__global__ __launch_bounds__(kBlock) void range_rows_pass2(
    const float *__restrict__ ws_min, const float *__restrict__ ws_max,
    float *__restrict__ ch_min, float *__restrict__ ch_max, int64_t c, int32_t groups,
    float qmax, float *__restrict__ scale, float *__restrict__ zero_point)
{
    const int64_t ic = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (ic >= c) return;
    float mn = __builtin_inff(), mx = -__builtin_inff();
    for (int32_t p = 0; p < groups; ++p) {
        mn = __builtin_fminf(mn, ws_min[(int64_t)p * c + ic]);
        mx = __builtin_fmaxf(mx, ws_max[(int64_t)p * c + ic]);
    }
    ch_min[ic] = mn;
    ch_max[ic] = mx;
    if (scale) {
        float sc, zp;
        prescale_one(mn, mx, qmax, sc, zp);
        scale[ic] = sc;
        zero_point[ic] = zp;
    }
}

// One wavefront per piece of an (n,c) slab at a time; scale and zero-point are
// wave-uniform.  `slabs` = N*C; a slab of hw elements has `chunks` pieces of chunk_len.
template <typename T>
__global__ __launch_bounds__(kBlock) void fq_fwd_rows(
    const void *x, void *x_hat, uint8_t *__restrict__ codes,
    const float *__restrict__ scale, const float *__restrict__ zero_point, float qmax,
    int64_t slabs, int64_t c, int64_t hw, int32_t chunks, int64_t chunk_len)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    const int64_t nwaves = (int64_t)gridDim.x * (kBlock / kWave);
    for (int64_t item = wave0; item < slabs * chunks; item += nwaves) {
        const int64_t slab = item / chunks, q = item % chunks;
        const int64_t ic = slab % c;
        const float s = scale[ic], z = zero_point[ic];
        const int64_t base = slab * hw;
        const int64_t k1 = (q + 1) * chunk_len < hw ? (q + 1) * chunk_len : hw;
        for (int64_t k = q * chunk_len + lane; k < k1; k += kWave) {
            float qv = clamp_code(raw_code(T::load1(x, base + k), s, z), qmax);
            if (x_hat) T::store1(x_hat, base + k, dequant(qv, s, z));
            if (codes) codes[base + k] = (uint8_t)qv;
        }
    }
}

template <typename T>
__global__ __launch_bounds__(kBlock) void fq_bwd_rows(
    const void *x, const void *dy, void *dx,
    const float *__restrict__ scale, const float *__restrict__ zero_point, float qmax,
    int64_t slabs, int64_t c, int64_t hw, int32_t chunks, int64_t chunk_len)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t wave0 = (int64_t)blockIdx.x * (kBlock / kWave) + threadIdx.x / kWave;
    const int64_t nwaves = (int64_t)gridDim.x * (kBlock / kWave);
    for (int64_t item = wave0; item < slabs * chunks; item += nwaves) {
        const int64_t slab = item / chunks, q = item % chunks;
        const int64_t ic = slab % c;
        const float s = scale[ic], z = zero_point[ic];
        const int64_t base = slab * hw;
        const int64_t k1 = (q + 1) * chunk_len < hw ? (q + 1) * chunk_len : hw;
        for (int64_t k = q * chunk_len + lane; k < k1; k += kWave) {
            bool keep = in_range(raw_code(T::load1(x, base + k), s, z), qmax);
            T::store_gated1(dx, dy, base + k, keep);
        }
    }
}

// ---------------------------------------------------------------------------
// prescale: Eq. 5 for all channels at once
// ---------------------------------------------------------------------------

__global__ __launch_bounds__(kBlock) void prescale_kernel(
    const float *__restrict__ ch_min, const float *__restrict__ ch_max, int64_t c, float qmax,
    float *__restrict__ scale, float *__restrict__ zero_point)
{
    const int64_t ic = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (ic >= c) return;
    float s, z;
    prescale_one(ch_min[ic], ch_max[ic], qmax, s, z);
    scale[ic] = s;
    zero_point[ic] = z;
}

// ---------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------

static bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

static granq_status_t check_desc(const granq_desc_t *d) {
    if (!d) return GRANQ_ERR_INVALID_ARG;
    if (d->n <= 0 || d->c <= 0 || d->h <= 0 || d->w <= 0) return GRANQ_ERR_INVALID_ARG;
    if (d->dtype != GRANQ_F32 && d->dtype != GRANQ_BF16 && d->dtype != GRANQ_F16) return GRANQ_ERR_UNSUPPORTED;
    // element count and every index must fit in int64 with room to spare
    const int64_t lim = (int64_t)1 << 40;
    if (d->n > lim || d->c >= ((int64_t)1 << 31) || d->h > lim || d->w > lim) return GRANQ_ERR_UNSUPPORTED;
    if (d->h * d->w > lim) return GRANQ_ERR_UNSUPPORTED;
    __int128 e = (__int128)d->n * d->c * (d->h * d->w);
    if (e > ((__int128)1 << 46)) return GRANQ_ERR_UNSUPPORTED;
    return GRANQ_OK;
}

static bool aligned_elem(const void *p, granq_dtype_t dt) {
    return ((uintptr_t)p & (dt == GRANQ_F32 ? 3u : 1u)) == 0;
}

// Grid of the row kernels: enough wavefronts to fill the chip, no more than slabs.
static uint32_t row_grid(int64_t slabs) {
    int64_t blocks = ceil_div(slabs, kBlock / kWave);
    int64_t cap = (int64_t)GRANQ_ROW_TARGET_BLOCKS * 4;
    return (uint32_t)(blocks < cap ? blocks : cap);
}

template <typename T, int V, int MODE>
static void launch_fwd_mode(const ColPlan &pl, const void *x, void *x_hat, void *extra, int kind,
                            const float *s, const float *z, float qmax, hipStream_t st) {
    using vec_t = typename T::vec_t;
    dim3 grid((uint32_t)pl.col_tiles, (uint32_t)pl.row_groups), block(kEBlock);
    auto xv = (const vec_t *)x;
    auto yv = (vec_t *)x_hat;
    if (kind == kCodes) launch_kernel((fq_fwd_cols<T, V, GRANQ_F_ROWS, MODE, kCodes>), grid, block, 0, st, xv, yv, extra, s, z, qmax, pl);
    else if (kind == kPacked) launch_kernel((fq_fwd_cols<T, V, GRANQ_F_ROWS, MODE, kPacked>), grid, block, 0, st, xv, yv, extra, s, z, qmax, pl);
    else if (kind == kPackedOnly) launch_kernel((fq_fwd_cols<T, V, GRANQ_F_ROWS, MODE, kPackedOnly>), grid, block, 0, st, xv, yv, extra, s, z, qmax, pl);
    else if (kind == kCodesOnly) launch_kernel((fq_fwd_cols<T, V, GRANQ_F_ROWS, MODE, kCodesOnly>), grid, block, 0, st, xv, yv, extra, s, z, qmax, pl);
    else launch_kernel((fq_fwd_cols<T, V, GRANQ_F_ROWS, MODE, kNoExtra>), grid, block, 0, st, xv, yv, extra, s, z, qmax, pl);
}

template <typename T, int V, int U>
static void launch_fwd_mask_cols(const ColPlan &pl, const void *x, void *x_hat, void *mask,
                                 const float *s, const float *z, float qmax, hipStream_t st) {
    using vec_t = typename T::vec_t;
    dim3 grid((uint32_t)pl.col_tiles, (uint32_t)pl.row_groups), block(kEBlock);
    auto xv = (const vec_t *)x;
    auto yv = (vec_t *)x_hat;
    if (pl.mode == kOne) launch_kernel((fq_fwd_cols<T, V, U, kOne, kMask>), grid, block, 0, st, xv, yv, mask, s, z, qmax, pl);
    else if (pl.mode == kTwo) launch_kernel((fq_fwd_cols<T, V, U, kTwo, kMask>), grid, block, 0, st, xv, yv, mask, s, z, qmax, pl);
    else launch_kernel((fq_fwd_cols<T, V, U, kEach, kMask>), grid, block, 0, st, xv, yv, mask, s, z, qmax, pl);
}

// kind: kNoExtra, kCodes (extra = codes) or kCodesOnly (extra = codes, x_hat unused)
template <typename T, int V>
static void launch_fwd_cols(const ColPlan &pl, const void *x, void *x_hat, void *extra, int kind,
                            const float *s, const float *z, float qmax, hipStream_t st) {
    if (pl.mode == kOne) launch_fwd_mode<T, V, kOne>(pl, x, x_hat, extra, kind, s, z, qmax, st);
    else if (pl.mode == kTwo) launch_fwd_mode<T, V, kTwo>(pl, x, x_hat, extra, kind, s, z, qmax, st);
    else launch_fwd_mode<T, V, kEach>(pl, x, x_hat, extra, kind, s, z, qmax, st);
}

template <typename T, int V>
static void launch_bwd_cols(const ColPlan &pl, const void *x, const void *dy, void *dx,
                            const float *s, const float *z, float qmax, hipStream_t st) {
    using vec_t = typename T::vec_t;
    dim3 grid((uint32_t)pl.col_tiles, (uint32_t)pl.row_groups), block(kEBlock);
    auto xv = (const vec_t *)x;
    auto gv = (const vec_t *)dy;
    auto ov = (vec_t *)dx;
    if (pl.fold > 1) {
        if (pl.mode == kOne)
            launch_kernel((fq_bwd_cols<T, V, GRANQ_B_ROWS, true, kOne>), grid, block, 0, st, xv, gv, ov, s, z, qmax, pl);
        else if (pl.mode == kTwo)
            launch_kernel((fq_bwd_cols<T, V, GRANQ_B_ROWS, true, kTwo>), grid, block, 0, st, xv, gv, ov, s, z, qmax, pl);
        else
            launch_kernel((fq_bwd_cols<T, V, GRANQ_B_ROWS, true, kEach>), grid, block, 0, st, xv, gv, ov, s, z, qmax, pl);
    } else if (pl.mode == kOne)
        launch_kernel((fq_bwd_cols<T, V, GRANQ_B_ROWS, false, kOne>), grid, block, 0, st, xv, gv, ov, s, z, qmax, pl);
    else if (pl.mode == kTwo)
        launch_kernel((fq_bwd_cols<T, V, GRANQ_B_ROWS, false, kTwo>), grid, block, 0, st, xv, gv, ov, s, z, qmax, pl);
    else
        launch_kernel((fq_bwd_cols<T, V, GRANQ_B_ROWS, false, kEach>), grid, block, 0, st, xv, gv, ov, s, z, qmax, pl);
}

template <typename T, int V>
static void launch_range_cols(const ColPlan &pl, const void *x, float *ws_min, float *ws_max,
                              const Pass1Extra &px, hipStream_t st) {
    using vec_t = typename T::vec_t;
    dim3 grid((uint32_t)pl.col_tiles, (uint32_t)pl.row_groups), block(kRBlock);
    size_t lds = (size_t)2 * pl.kmax * sizeof(uint32_t);
    auto xv = (const vec_t *)x;
    if (pl.mode == kOne)
        launch_kernel((range_cols_pass1<T, V, kOne>), grid, block, lds, st, xv, ws_min, ws_max, pl, px);
    else if (pl.mode == kTwo)
        launch_kernel((range_cols_pass1<T, V, kTwo>), grid, block, lds, st, xv, ws_min, ws_max, pl, px);
    else
        launch_kernel((range_cols_pass1<T, V, kEach>), grid, block, lds, st, xv, ws_min, ws_max, pl, px);
}

static void launch_range_cols_any(const granq_desc_t *desc, const ColPlan &pl, const void *x, float *ws_min,
                                  float *ws_max, const Pass1Extra &px, hipStream_t st) {
    if (desc->dtype == GRANQ_F32) launch_range_cols<F32, GRANQ_R_V_F32>(pl, x, ws_min, ws_max, px, st);
    else if (desc->dtype == GRANQ_BF16) launch_range_cols<BF16, GRANQ_R_V_BF16>(pl, x, ws_min, ws_max, px, st);
    else launch_range_cols<F16, GRANQ_R_V_BF16>(pl, x, ws_min, ws_max, px, st);
}

// The forward that finishes the reduction: grid = finisher rows, then the forward's own rows.
template <typename T, int V, int MODE>
static void launch_fwd_finish_mode(const ColPlan &pl, const void *x, void *x_hat, void *extra, int kind,
                                   float qmax, const FinishArgs &fa, hipStream_t st) {
    using vec_t = typename T::vec_t;
    dim3 grid((uint32_t)pl.col_tiles, (uint32_t)(pl.row_groups + fa.finisher_rows)), block(kEBlock);
    auto xv = (const vec_t *)x;
    auto yv = (vec_t *)x_hat;
    if (kind == kCodes) launch_kernel((fq_fwd_finish_cols<T, V, GRANQ_F_ROWS, MODE, kCodes>), grid, block, 0, st, xv, yv, extra, qmax, pl, fa);
    else if (kind == kCodesOnly) launch_kernel((fq_fwd_finish_cols<T, V, GRANQ_F_ROWS, MODE, kCodesOnly>), grid, block, 0, st, xv, yv, extra, qmax, pl, fa);
    else launch_kernel((fq_fwd_finish_cols<T, V, GRANQ_F_ROWS, MODE, kNoExtra>), grid, block, 0, st, xv, yv, extra, qmax, pl, fa);
}

template <typename T, int V>
static void launch_fwd_finish(const ColPlan &pl, const void *x, void *x_hat, void *extra, int kind,
                              float qmax, const FinishArgs &fa, hipStream_t st) {
    if (pl.mode == kOne) launch_fwd_finish_mode<T, V, kOne>(pl, x, x_hat, extra, kind, qmax, fa, st);
    else if (pl.mode == kTwo) launch_fwd_finish_mode<T, V, kTwo>(pl, x, x_hat, extra, kind, qmax, fa, st);
    else launch_fwd_finish_mode<T, V, kEach>(pl, x, x_hat, extra, kind, qmax, fa, st);
}

// Argument checks of the forward; scale / zero_point may be vectors it will be given later.
static granq_status_t fwd_check(const void *x, const granq_desc_t *desc, const float *scale,
                                const float *zero_point, int bits, const void *x_hat,
                                const uint8_t *codes_or_null) {
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    if (!x || !scale || !zero_point) return GRANQ_ERR_INVALID_ARG;
    if (!x_hat && !codes_or_null) return GRANQ_ERR_INVALID_ARG;      // nothing to write
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (!aligned_elem(x, desc->dtype) || (x_hat && !aligned_elem(x_hat, desc->dtype)) ||
        !aligned_elem(scale, GRANQ_F32) || !aligned_elem(zero_point, GRANQ_F32))
        return GRANQ_ERR_UNSUPPORTED;
    return GRANQ_OK;
}

// The 128-bit column kernels of the forward apply: plan, pointers, packed-code alignment
// (codes are stored VEC bytes at a time).
static bool fwd_cols_ok(const ColPlan &cp, const granq_desc_t *desc, const void *x, const void *x_hat,
                        const uint8_t *codes_or_null) {
    const bool codes_ok = !codes_or_null || ((uintptr_t)codes_or_null % (size_t)vec_of(desc->dtype)) == 0;
    return cp.ok && aligned16(x) && (!x_hat || aligned16(x_hat)) && codes_ok;
}

}  // namespace granq

using namespace granq;

extern "C" {

const char *granq_status_string(granq_status_t status) {
    switch (status) {
        case GRANQ_OK: return "GRANQ_OK";
        case GRANQ_ERR_INVALID_ARG: return "GRANQ_ERR_INVALID_ARG: null pointer, non-positive dimension or bits outside 1..8";
        case GRANQ_ERR_UNSUPPORTED: return "GRANQ_ERR_UNSUPPORTED: unknown dtype, misaligned pointer or tensor too large";
        case GRANQ_ERR_WORKSPACE: return "GRANQ_ERR_WORKSPACE: workspace missing, misaligned or too small";
        case GRANQ_ERR_HIP: return "GRANQ_ERR_HIP: the HIP runtime rejected a launch";
    }
    return "GRANQ: unknown status";
}

const char *granq_version(void) { return "granq-gfx950 0.1"; }

granq_status_t granq_workspace_bytes(const granq_desc_t *desc, size_t *bytes_out) {
    if (!bytes_out) return GRANQ_ERR_INVALID_ARG;
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    const int64_t hw = desc->h * desc->w;
    RowPlan rp = make_row_plan(desc->n, desc->c, hw);
    size_t bytes = 2 * (size_t)rp.row_groups * (size_t)rp.chunks * (size_t)desc->c * sizeof(float);
    ColPlan cp = range_plan(desc);
    if (cp.ok && col_ws_bytes(cp) > bytes) bytes = col_ws_bytes(cp);
    *bytes_out = bytes;
    return GRANQ_OK;
}

granq_status_t granq_plan_describe(const granq_desc_t *desc, int64_t out[24]) {
    if (!out) return GRANQ_ERR_INVALID_ARG;
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    ColPlan cp = range_plan(desc);
    out[0] = cp.ok ? 1 : 0;
    out[1] = cp.rows;
    out[2] = cp.row_len;
    out[3] = cp.hw;
    out[4] = cp.span;
    out[5] = cp.col_tiles;
    out[6] = cp.row_groups;
    out[7] = cp.rows_per_group;
    out[8] = cp.kmax;
    out[9] = cp.uniform ? 1 : 0;
    out[10] = cp.hw_div.m;
    out[11] = cp.hw_div.s1;
    out[12] = cp.hw_div.s2;
    ColPlan fp = fwd_plan(desc), bp = bwd_plan(desc);
    out[13] = fp.rows_per_group;
    out[14] = bp.rows_per_group;
    out[15] = fp.span;
    out[16] = cp.fold;
    out[17] = one_call_forward_launches(desc);
    out[18] = !cp.ok ? 2 : (direct_channels(cp) > 0 ? 1 : 2);
    for (int i = 19; i < 24; ++i) out[i] = 0;
    return GRANQ_OK;
}

// Argument checks of the reduction (nothing is launched on a refusal).
static granq_status_t range_check(const void *x, const granq_desc_t *desc, const float *ch_min,
                                  const float *ch_max, const void *workspace, size_t workspace_bytes) {
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    if (!x || !ch_min || !ch_max) return GRANQ_ERR_INVALID_ARG;
    if (!aligned_elem(x, desc->dtype) || !aligned_elem(ch_min, GRANQ_F32) || !aligned_elem(ch_max, GRANQ_F32))
        return GRANQ_ERR_UNSUPPORTED;
    size_t need = 0;
    granq_workspace_bytes(desc, &need);
    if (!workspace || workspace_bytes < need || !aligned16(workspace)) return GRANQ_ERR_WORKSPACE;
    return GRANQ_OK;
}

static void launch_range_pass2(const ColPlan &cp, const float *ws_min, const float *ws_max, float *ch_min,
                               float *ch_max, float qmax, float *scale, float *zero_point, hipStream_t hs) {
    dim3 block(kBlock);
    if (partials_per_channel(cp) > 512) {
        dim3 grid((uint32_t)cp.channels);
        launch_kernel(range_cols_pass2<kBlock / kWave>, grid, block, 0, hs, ws_min, ws_max, ch_min, ch_max, cp,
                      qmax, scale, zero_point);
    } else {
        dim3 grid((uint32_t)ceil_div(cp.channels, kBlock / kWave));
        launch_kernel(range_cols_pass2<1>, grid, block, 0, hs, ws_min, ws_max, ch_min, ch_max, cp,
                      qmax, scale, zero_point);
    }
}

// Ranges, and with non-null `scale` / `zero_point` also Eq. 5: two launches, or one where the
// first pass already holds every channel whole.
static granq_status_t range_impl(const void *x, const granq_desc_t *desc, float *ch_min,
                                 float *ch_max, float qmax, float *scale, float *zero_point,
                                 void *workspace, size_t workspace_bytes, void *stream) {
    granq_status_t st = range_check(x, desc, ch_min, ch_max, workspace, workspace_bytes);
    if (st != GRANQ_OK) return st;
    hipStream_t hs = (hipStream_t)stream;
    const int64_t hw = desc->h * desc->w;
    ColPlan cp = range_plan(desc);
    if (cp.ok && aligned16(x)) {
        const size_t floats = col_ws_floats(cp);
        float *ws_min = (float *)workspace;
        float *ws_max = ws_min + floats;
        Pass1Extra px{};
        px.direct = direct_channels(cp);
        px.ch_min = ch_min;
        px.ch_max = ch_max;
        px.scale = scale;
        px.zero_point = zero_point;
        px.qmax = qmax;
        launch_range_cols_any(desc, cp, x, ws_min, ws_max, px, hs);
        if (px.direct > 0) return launched();
        st = launched();
        if (st != GRANQ_OK) return st;
        launch_range_pass2(cp, ws_min, ws_max, ch_min, ch_max, qmax, scale, zero_point, hs);
        return launched();
    }
    RowPlan rp = make_row_plan(desc->n, desc->c, hw);
    const int64_t per_channel = (int64_t)rp.row_groups * rp.chunks;
    const size_t floats = (size_t)per_channel * (size_t)desc->c;
    float *ws_min = (float *)workspace;
    float *ws_max = ws_min + floats;
    dim3 grid((uint32_t)(desc->c * per_channel)), block(kBlock);
    if (desc->dtype == GRANQ_F32)
        launch_kernel(range_rows_pass1<F32>, grid, block, 0, hs, x, ws_min, ws_max, desc->n, desc->c, hw, rp);
    else if (desc->dtype == GRANQ_BF16)
        launch_kernel(range_rows_pass1<BF16>, grid, block, 0, hs, x, ws_min, ws_max, desc->n, desc->c, hw, rp);
    else
        launch_kernel(range_rows_pass1<F16>, grid, block, 0, hs, x, ws_min, ws_max, desc->n, desc->c, hw, rp);
    st = launched();
    if (st != GRANQ_OK) return st;
    dim3 grid2((uint32_t)ceil_div(desc->c, kBlock));
    launch_kernel(range_rows_pass2, grid2, block, 0, hs, ws_min, ws_max, ch_min, ch_max, desc->c, (int32_t)per_channel,
                       qmax, scale, zero_point);
    return launched();
}

granq_status_t granq_range_reduce(const void *x, const granq_desc_t *desc, float *ch_min,
                                  float *ch_max, void *workspace, size_t workspace_bytes,
                                  void *stream) {
    return range_impl(x, desc, ch_min, ch_max, 0.0f, nullptr, nullptr, workspace, workspace_bytes, stream);
}

// Library-owned scratch for callers that cannot bring a workspace (see granq.h).  One copy of
// the array lives on every GPU the library is loaded on; in host code its name is only a
// handle for hipGetSymbolAddress, never an address a kernel could use.
static __device__ __align__(256) unsigned char scratch[GRANQ_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
static std::atomic<void *> scratch_of_device[kMaxDevices];

// Device address of the current device's copy of `scratch`, resolved once per device.
static granq_status_t static_scratch(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GRANQ_ERR_HIP;
    void *p = scratch_of_device[dev].load(std::memory_order_acquire);
    if (!p) {
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return GRANQ_ERR_HIP;
        scratch_of_device[dev].store(p, std::memory_order_release);   // same value from every thread
    }
    *out = p;
    return GRANQ_OK;
}

granq_status_t granq_range_reduce_noalloc(const void *x, const granq_desc_t *desc, float *ch_min,
                                          float *ch_max, void *stream) {
    size_t need = 0;
    granq_status_t st = granq_workspace_bytes(desc, &need);
    if (st != GRANQ_OK) return st;
    if (need > GRANQ_STATIC_SCRATCH_BYTES) return GRANQ_ERR_WORKSPACE;
    void *ws = nullptr;
    st = static_scratch(&ws);
    if (st != GRANQ_OK) return st;
    // every partial the second pass reads is written by the first pass of the same call:
    // nothing in the scratch has to start at zero
    return range_impl(x, desc, ch_min, ch_max, 0.0f, nullptr, nullptr, ws, GRANQ_STATIC_SCRATCH_BYTES, stream);
}

granq_status_t granq_calibrate(const void *x, const granq_desc_t *desc, int bits, float *ch_min,
                               float *ch_max, float *scale, float *zero_point, void *workspace,
                               size_t workspace_bytes, void *stream) {
    if (!scale || !zero_point) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (!aligned_elem(scale, GRANQ_F32) || !aligned_elem(zero_point, GRANQ_F32)) return GRANQ_ERR_UNSUPPORTED;
    return range_impl(x, desc, ch_min, ch_max, (float)((1 << bits) - 1), scale, zero_point,
                      workspace, workspace_bytes, stream);
}

}  // extern "C"

namespace granq {

// The two-launch form can be compiled out (-DGRANQ_TWO_LAUNCH=0) to measure it against three.
#ifndef GRANQ_TWO_LAUNCH
#define GRANQ_TWO_LAUNCH 1
#endif

// Polls of a hand-over slot before a waiting wavefront of the finishing forward computes the
// parameters itself (about a microsecond each).  GRANQ_SPIN_LIMIT in the environment
// overrides it; tests set it to 0 so that every waiting wavefront takes that path.
// Small tensors with large maps do not wait at all: their launch is over in a few microseconds, of
// which the finishers' gather -> Eq. 5 -> publish -> poll chain is two to three, while a wavefront
// that gathers its own channel's partials (from the caches) loses about one.  Elsewhere the order
// reverses: on large tensors thousands of blocks would each repeat the gather, and where a
// wavefront's row of vectors spans many channels (7 x 7 maps) it would gather them one by one.
#ifndef GRANQ_SELF_DERIVE_MAX_BYTES
#define GRANQ_SELF_DERIVE_MAX_BYTES (24u << 20)
#endif
static int32_t spin_limit(const granq_desc_t *desc = nullptr) {
    const char *e = getenv("GRANQ_SPIN_LIMIT");
    if (e && *e) {
        const long v = strtol(e, nullptr, 10);
        return (int32_t)(v < 0 ? 0 : (v > (1 << 24) ? (1 << 24) : v));
    }
    if (desc) {
        const int64_t wave_span = (int64_t)kWave * (desc->dtype == GRANQ_F32 ? 4 : 8);   // elements of one vector per lane
        if (tensor_bytes(desc) <= (int64_t)GRANQ_SELF_DERIVE_MAX_BYTES && desc->h * desc->w >= wave_span) return 0;
    }
    return 20000;
}

bool two_launches_apply(const void *x, const granq_desc_t *desc, const void *x_hat,
                        const uint8_t *codes_or_null) {
    if (!GRANQ_TWO_LAUNCH || check_desc(desc) != GRANQ_OK) return false;
    const ColPlan cp = range_plan(desc), fp = fwd_plan(desc);
    if (!cp.ok || !x || !aligned16(x) || !fwd_cols_ok(fp, desc, x, x_hat, codes_or_null)) return false;
    // the first pass alone is final, or a channel has more partials than one wavefront should gather
    if (direct_channels(cp) > 0 || partials_per_channel(cp) > 512) return false;
    return fp.row_groups + finisher_rows_of(cp, fp) <= 65535;
}

// Alg. 1 up to the accumulation in two launches for tensors on the 128-bit column path:
// the first pass of the reduction, then the forward, whose leading blocks finish the
// reduction (second pass and Eq. 5) and hand scale and zero-point to the others through the
// workspace.
granq_status_t calibrate_fwd_two_launches(const void *x, const granq_desc_t *desc, int bits, float *ch_min,
                                          float *ch_max, float *scale, float *zero_point, void *x_hat,
                                          uint8_t *codes_or_null, void *workspace, size_t workspace_bytes,
                                          void *stream) {
    const ColPlan cp = range_plan(desc), fp = fwd_plan(desc);
    const int64_t finisher_rows = finisher_rows_of(cp, fp);
    // the checks of granq_calibrate and of granq_fakequant_fwd, all before the first launch
    if (!scale || !zero_point) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (!aligned_elem(scale, GRANQ_F32) || !aligned_elem(zero_point, GRANQ_F32)) return GRANQ_ERR_UNSUPPORTED;
    granq_status_t st = range_check(x, desc, ch_min, ch_max, workspace, workspace_bytes);
    if (st != GRANQ_OK) return st;
    st = fwd_check(x, desc, scale, zero_point, bits, x_hat, codes_or_null);
    if (st != GRANQ_OK) return st;

    hipStream_t hs = (hipStream_t)stream;
    const float qmax = (float)((1 << bits) - 1);
    float *ws_min = (float *)workspace;
    float *ws_max = ws_min + col_ws_floats(cp);
    uint64_t *params = (uint64_t *)((char *)workspace + col_params_offset(cp));
    Pass1Extra px{};
    px.params = params;
    launch_range_cols_any(desc, cp, x, ws_min, ws_max, px, hs);
    st = launched();
    if (st != GRANQ_OK) return st;
    FinishArgs fa{};
    fa.ws_min = ws_min;
    fa.ws_max = ws_max;
    fa.params = params;
    fa.ch_min = ch_min;
    fa.ch_max = ch_max;
    fa.scale = scale;
    fa.zero_point = zero_point;
    fa.rplan = cp;
    fa.finisher_rows = (int32_t)finisher_rows;
    fa.spin_limit = spin_limit(desc);
    const int kind = !x_hat ? kCodesOnly : (codes_or_null ? kCodes : kNoExtra);
    if (desc->dtype == GRANQ_F32) launch_fwd_finish<F32, GRANQ_E_V_F32>(fp, x, x_hat, codes_or_null, kind, qmax, fa, hs);
    else if (desc->dtype == GRANQ_BF16) launch_fwd_finish<BF16, GRANQ_E_V_BF16>(fp, x, x_hat, codes_or_null, kind, qmax, fa, hs);
    else launch_fwd_finish<F16, GRANQ_E_V_BF16>(fp, x, x_hat, codes_or_null, kind, qmax, fa, hs);
    return launched();
}

}  // namespace granq

extern "C" {

granq_status_t granq_prescale(const float *ch_min, const float *ch_max, int64_t c, int bits,
                              float *scale, float *zero_point, void *stream) {
    if (!ch_min || !ch_max || !scale || !zero_point) return GRANQ_ERR_INVALID_ARG;
    if (c <= 0 || bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (c >= ((int64_t)1 << 31)) return GRANQ_ERR_UNSUPPORTED;
    if (!aligned_elem(ch_min, GRANQ_F32) || !aligned_elem(ch_max, GRANQ_F32) ||
        !aligned_elem(scale, GRANQ_F32) || !aligned_elem(zero_point, GRANQ_F32))
        return GRANQ_ERR_UNSUPPORTED;
    const float qmax = (float)((1 << bits) - 1);
    dim3 grid((uint32_t)ceil_div(c, kBlock)), block(kBlock);
    launch_kernel(prescale_kernel, grid, block, 0, (hipStream_t)stream, ch_min, ch_max, c, qmax, scale, zero_point);
    return launched();
}

granq_status_t granq_fakequant_fwd(const void *x, const granq_desc_t *desc, const float *scale,
                                   const float *zero_point, int bits, void *x_hat,
                                   uint8_t *codes_or_null, void *stream) {
    granq_status_t st = fwd_check(x, desc, scale, zero_point, bits, x_hat, codes_or_null);
    if (st != GRANQ_OK) return st;
    const float qmax = (float)((1 << bits) - 1);
    hipStream_t hs = (hipStream_t)stream;
    ColPlan cp = fwd_plan(desc);
    if (fwd_cols_ok(cp, desc, x, x_hat, codes_or_null)) {
        const int kind = !x_hat ? kCodesOnly : (codes_or_null ? kCodes : kNoExtra);
        if (desc->dtype == GRANQ_F32) launch_fwd_cols<F32, GRANQ_E_V_F32>(cp, x, x_hat, codes_or_null, kind, scale, zero_point, qmax, hs);
        else if (desc->dtype == GRANQ_BF16) launch_fwd_cols<BF16, GRANQ_E_V_BF16>(cp, x, x_hat, codes_or_null, kind, scale, zero_point, qmax, hs);
        else launch_fwd_cols<F16, GRANQ_E_V_BF16>(cp, x, x_hat, codes_or_null, kind, scale, zero_point, qmax, hs);
        return launched();
    }
    const int64_t hw = desc->h * desc->w;
    const int64_t slabs = desc->n * desc->c;
    const RowPlan rp = make_row_plan(desc->n, desc->c, hw);
    dim3 grid(row_grid(slabs * rp.chunks)), block(kBlock);
    if (desc->dtype == GRANQ_F32)
        launch_kernel(fq_fwd_rows<F32>, grid, block, 0, hs, x, x_hat, codes_or_null, scale, zero_point, qmax, slabs, desc->c, hw, rp.chunks, rp.chunk_len);
    else if (desc->dtype == GRANQ_BF16)
        launch_kernel(fq_fwd_rows<BF16>, grid, block, 0, hs, x, x_hat, codes_or_null, scale, zero_point, qmax, slabs, desc->c, hw, rp.chunks, rp.chunk_len);
    else
        launch_kernel(fq_fwd_rows<F16>, grid, block, 0, hs, x, x_hat, codes_or_null, scale, zero_point, qmax, slabs, desc->c, hw, rp.chunks, rp.chunk_len);
    return launched();
}

granq_status_t granq_packed4_bytes(const granq_desc_t *desc, size_t *bytes_out) {
    if (!bytes_out) return GRANQ_ERR_INVALID_ARG;
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    *bytes_out = (size_t)((desc->n * desc->c * desc->h * desc->w + 1) / 2);
    return GRANQ_OK;
}

granq_status_t granq_fakequant_fwd_packed4(const void *x, const granq_desc_t *desc, const float *scale,
                                           const float *zero_point, int bits, void *x_hat_or_null,
                                           uint8_t *packed, void *stream) {
    if (!packed) return GRANQ_ERR_INVALID_ARG;
    granq_status_t st = fwd_check(x, desc, scale, zero_point, bits, x_hat_or_null, packed);
    if (st != GRANQ_OK) return st;
    if (bits > 4) return GRANQ_ERR_INVALID_ARG;                     // a code must fit a nibble
    const float qmax = (float)((1 << bits) - 1);
    hipStream_t hs = (hipStream_t)stream;
    ColPlan cp = fwd_plan(desc);
    // a lane stores the nibbles of one vector at once: 2 bytes (float32) or 4 (16-bit types)
    const bool packed_ok = ((uintptr_t)packed % (size_t)(vec_of(desc->dtype) / 2)) == 0;
    if (cp.ok && aligned16(x) && (!x_hat_or_null || aligned16(x_hat_or_null)) && packed_ok) {
        const int kind = x_hat_or_null ? kPacked : kPackedOnly;
        if (desc->dtype == GRANQ_F32) launch_fwd_cols<F32, GRANQ_E_V_F32>(cp, x, x_hat_or_null, packed, kind, scale, zero_point, qmax, hs);
        else if (desc->dtype == GRANQ_BF16) launch_fwd_cols<BF16, GRANQ_E_V_BF16>(cp, x, x_hat_or_null, packed, kind, scale, zero_point, qmax, hs);
        else launch_fwd_cols<F16, GRANQ_E_V_BF16>(cp, x, x_hat_or_null, packed, kind, scale, zero_point, qmax, hs);
        return launched();
    }
    const int64_t hw = desc->h * desc->w;
    const int64_t total = desc->n * desc->c * hw;
    const int64_t want = ceil_div(ceil_div(total, 2), kBlock);
    dim3 grid((uint32_t)(want < GRANQ_ROW_TARGET_BLOCKS * 4 ? want : GRANQ_ROW_TARGET_BLOCKS * 4)), block(kBlock);
    if (desc->dtype == GRANQ_F32)
        launch_kernel(fwd_packed_bytes<F32>, grid, block, 0, hs, x, x_hat_or_null, scale, zero_point, qmax, desc->c, hw, total, packed);
    else if (desc->dtype == GRANQ_BF16)
        launch_kernel(fwd_packed_bytes<BF16>, grid, block, 0, hs, x, x_hat_or_null, scale, zero_point, qmax, desc->c, hw, total, packed);
    else
        launch_kernel(fwd_packed_bytes<F16>, grid, block, 0, hs, x, x_hat_or_null, scale, zero_point, qmax, desc->c, hw, total, packed);
    return launched();
}

granq_status_t granq_fakequant_bwd(const void *x, const void *dy, const granq_desc_t *desc,
                                   const float *scale, const float *zero_point, int bits,
                                   void *dx, void *stream) {
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    if (!x || !dy || !dx || !scale || !zero_point) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (!aligned_elem(x, desc->dtype) || !aligned_elem(dy, desc->dtype) || !aligned_elem(dx, desc->dtype) ||
        !aligned_elem(scale, GRANQ_F32) || !aligned_elem(zero_point, GRANQ_F32))
        return GRANQ_ERR_UNSUPPORTED;
    const float qmax = (float)((1 << bits) - 1);
    hipStream_t hs = (hipStream_t)stream;
    ColPlan cp = bwd_plan(desc);
    if (cp.ok && aligned16(x) && aligned16(dy) && aligned16(dx)) {
        if (desc->dtype == GRANQ_F32) launch_bwd_cols<F32, GRANQ_E_V_F32>(cp, x, dy, dx, scale, zero_point, qmax, hs);
        else if (desc->dtype == GRANQ_BF16) launch_bwd_cols<BF16, GRANQ_E_V_BF16>(cp, x, dy, dx, scale, zero_point, qmax, hs);
        else launch_bwd_cols<F16, GRANQ_E_V_BF16>(cp, x, dy, dx, scale, zero_point, qmax, hs);
        return launched();
    }
    const int64_t hw = desc->h * desc->w;
    const int64_t slabs = desc->n * desc->c;
    const RowPlan rp = make_row_plan(desc->n, desc->c, hw);
    dim3 grid(row_grid(slabs * rp.chunks)), block(kBlock);
    if (desc->dtype == GRANQ_F32)
        launch_kernel(fq_bwd_rows<F32>, grid, block, 0, hs, x, dy, dx, scale, zero_point, qmax, slabs, desc->c, hw, rp.chunks, rp.chunk_len);
    else if (desc->dtype == GRANQ_BF16)
        launch_kernel(fq_bwd_rows<BF16>, grid, block, 0, hs, x, dy, dx, scale, zero_point, qmax, slabs, desc->c, hw, rp.chunks, rp.chunk_len);
    else
        launch_kernel(fq_bwd_rows<F16>, grid, block, 0, hs, x, dy, dx, scale, zero_point, qmax, slabs, desc->c, hw, rp.chunks, rp.chunk_len);
    return launched();
}

// The vectorised mask kernels need whole bytes per lane pair: rows that are a multiple of
// eight elements (and, as everywhere, 16-byte vectors).
static bool mask_vector_ok(const ColPlan &cp) {
    return cp.ok && cp.row_len % 8 == 0;
}

granq_status_t granq_mask_bytes(const granq_desc_t *desc, size_t *bytes_out) {
    if (!bytes_out) return GRANQ_ERR_INVALID_ARG;
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    *bytes_out = (size_t)((desc->n * desc->c * desc->h * desc->w + 7) / 8);
    return GRANQ_OK;
}

granq_status_t granq_fakequant_fwd_mask(const void *x, const granq_desc_t *desc, const float *scale,
                                        const float *zero_point, int bits, void *x_hat,
                                        uint8_t *mask, void *stream) {
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    if (!x || !x_hat || !scale || !zero_point || !mask) return GRANQ_ERR_INVALID_ARG;
    if (bits < 1 || bits > 8) return GRANQ_ERR_INVALID_ARG;
    if (!aligned_elem(x, desc->dtype) || !aligned_elem(x_hat, desc->dtype) ||
        !aligned_elem(scale, GRANQ_F32) || !aligned_elem(zero_point, GRANQ_F32))
        return GRANQ_ERR_UNSUPPORTED;
    const float qmax = (float)((1 << bits) - 1);
    hipStream_t hs = (hipStream_t)stream;
    ColPlan cp = fwd_mask_plan(desc);
    if (mask_vector_ok(cp) && aligned16(x) && aligned16(x_hat)) {
        if (desc->dtype == GRANQ_F32) launch_fwd_mask_cols<F32, GRANQ_M_V_F32, GRANQ_M_ROWS_F32>(cp, x, x_hat, mask, scale, zero_point, qmax, hs);
        else if (desc->dtype == GRANQ_BF16) launch_fwd_mask_cols<BF16, GRANQ_M_V_BF16, GRANQ_M_ROWS_BF16>(cp, x, x_hat, mask, scale, zero_point, qmax, hs);
        else launch_fwd_mask_cols<F16, GRANQ_M_V_BF16, GRANQ_M_ROWS_BF16>(cp, x, x_hat, mask, scale, zero_point, qmax, hs);
        return launched();
    }
    // any other shape or alignment: gate bits from x first (x_hat may alias x), then the forward
    const int64_t hw = desc->h * desc->w;
    const int64_t total = desc->n * desc->c * hw;
    const int64_t want = ceil_div(ceil_div(total, 8), kBlock);
    dim3 grid((uint32_t)(want < GRANQ_ROW_TARGET_BLOCKS * 4 ? want : GRANQ_ROW_TARGET_BLOCKS * 4)), block(kBlock);
    if (desc->dtype == GRANQ_F32)
        launch_kernel(mask_from_x_bytes<F32>, grid, block, 0, hs, x, scale, zero_point, qmax, desc->c, hw, total, mask);
    else if (desc->dtype == GRANQ_BF16)
        launch_kernel(mask_from_x_bytes<BF16>, grid, block, 0, hs, x, scale, zero_point, qmax, desc->c, hw, total, mask);
    else
        launch_kernel(mask_from_x_bytes<F16>, grid, block, 0, hs, x, scale, zero_point, qmax, desc->c, hw, total, mask);
    st = launched();
    if (st != GRANQ_OK) return st;
    return granq_fakequant_fwd(x, desc, scale, zero_point, bits, x_hat, nullptr, stream);
}

granq_status_t granq_fakequant_bwd_mask(const void *dy, const uint8_t *mask, const granq_desc_t *desc,
                                        void *dx, void *stream) {
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    if (!dy || !mask || !dx) return GRANQ_ERR_INVALID_ARG;
    if (!aligned_elem(dy, desc->dtype) || !aligned_elem(dx, desc->dtype)) return GRANQ_ERR_UNSUPPORTED;
    hipStream_t hs = (hipStream_t)stream;
    ColPlan cp = bwd_plan(desc);
    // fq_bwd_mask_cols handles one vector per lane
    if (mask_vector_ok(cp) && GRANQ_E_V_F32 == 1 && GRANQ_E_V_BF16 == 1 && aligned16(dy) && aligned16(dx)) {
        dim3 grid((uint32_t)cp.col_tiles, (uint32_t)cp.row_groups), block(kEBlock);
        const bool nt = cp.nt_row_end > 0;
        if (desc->dtype == GRANQ_F32) {
            if (nt) launch_kernel((fq_bwd_mask_cols<F32, GRANQ_B_ROWS, true>), grid, block, 0, hs, (const F32::vec_t *)dy, mask, (F32::vec_t *)dx, cp);
            else launch_kernel((fq_bwd_mask_cols<F32, GRANQ_B_ROWS, false>), grid, block, 0, hs, (const F32::vec_t *)dy, mask, (F32::vec_t *)dx, cp);
        } else {
            // gating moves 16-bit patterns without interpreting them: one kernel for both 16-bit types
            if (nt) launch_kernel((fq_bwd_mask_cols<Pack16, GRANQ_B_ROWS, true>), grid, block, 0, hs, (const Pack16::vec_t *)dy, mask, (Pack16::vec_t *)dx, cp);
            else launch_kernel((fq_bwd_mask_cols<Pack16, GRANQ_B_ROWS, false>), grid, block, 0, hs, (const Pack16::vec_t *)dy, mask, (Pack16::vec_t *)dx, cp);
        }
        return launched();
    }
    const int64_t total = desc->n * desc->c * desc->h * desc->w;
    const int64_t want = ceil_div(ceil_div(total, 8), kBlock);
    dim3 grid((uint32_t)(want < GRANQ_ROW_TARGET_BLOCKS * 4 ? want : GRANQ_ROW_TARGET_BLOCKS * 4)), block(kBlock);
    if (desc->dtype == GRANQ_F32) launch_kernel(bwd_mask_bytes<F32>, grid, block, 0, hs, dy, mask, total, dx);
    else launch_kernel(bwd_mask_bytes<Pack16>, grid, block, 0, hs, dy, mask, total, dx);
    return launched();
}

}  // extern "C"

// ---- single-launch ("resident") form --------------------------------------------------------

namespace granq {

__global__ __launch_bounds__(kBlock) void zero_words(uint32_t *p, size_t words) {
    for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < words; i += (size_t)gridDim.x * kBlock) p[i] = 0u;
}

template <typename T, int R>
static hipError_t launch_resident(const ColPlan &pl, const ResidentArgs &ra, hipStream_t st, int *blocks_per_cu) {
    dim3 grid((uint32_t)pl.col_tiles, (uint32_t)pl.row_groups), block(kResBlock);
    const size_t lds = (size_t)2 * pl.kmax * sizeof(uint32_t);
    void (*kernel)(ResidentArgs) = pl.mode == kOne ? fq_resident_cols<T, R, kOne>
                                 : (pl.mode == kTwo ? fq_resident_cols<T, R, kTwo> : fq_resident_cols<T, R, kEach>);
    // all blocks must fit the chip together for this form to be worth taking
    hipError_t e = hipOccupancyMaxActiveBlocksPerMultiprocessor(blocks_per_cu, (const void *)kernel, kResBlock, lds);
    if (e != hipSuccess) return e;
    int dev = 0, cus = 0;
    if ((e = hipGetDevice(&dev)) != hipSuccess) return e;
    if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return e;
    if ((int64_t)pl.col_tiles * pl.row_groups > (int64_t)*blocks_per_cu * cus) {
        *blocks_per_cu = -1;
        return hipSuccess;
    }
    launch_kernel(kernel, grid, block, lds, st, ra);
    return hipSuccess;
}

}  // namespace granq

extern "C" {

granq_status_t granq_resident_state_bytes(const granq_desc_t *desc, size_t *bytes_out) {
    if (!bytes_out) return GRANQ_ERR_INVALID_ARG;
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    const ResidentPlan rp = resident_plan(desc);
    if (!rp.ok) return GRANQ_ERR_UNSUPPORTED;
    *bytes_out = rp.bytes;
    return GRANQ_OK;
}

granq_status_t granq_resident_state_init(void *state, size_t state_bytes, void *stream) {
    if (!state || state_bytes == 0) return GRANQ_ERR_INVALID_ARG;
    if (!aligned16(state) || state_bytes % 4 != 0) return GRANQ_ERR_UNSUPPORTED;
    const size_t words = state_bytes / 4;
    const size_t blocks = (words + kBlock - 1) / kBlock;
    launch_kernel(zero_words, dim3((uint32_t)(blocks < 4096 ? blocks : 4096)), dim3(kBlock), 0, (hipStream_t)stream,
                  (uint32_t *)state, words);
    return launched();
}

granq_status_t granq_calibrate_fakequant_fwd_resident(const void *x, const granq_desc_t *desc, int bits,
                                                      float *ch_min, float *ch_max, float *scale,
                                                      float *zero_point, void *x_hat, uint8_t *codes_or_null,
                                                      void *state, size_t state_bytes, void *stream) {
    granq_status_t st = check_desc(desc);
    if (st != GRANQ_OK) return st;
    if (!ch_min || !ch_max || !scale || !zero_point) return GRANQ_ERR_INVALID_ARG;
    st = fwd_check(x, desc, scale, zero_point, bits, x_hat, codes_or_null);
    if (st != GRANQ_OK) return st;
    if (!aligned_elem(ch_min, GRANQ_F32) || !aligned_elem(ch_max, GRANQ_F32)) return GRANQ_ERR_UNSUPPORTED;
    const ResidentPlan rp = resident_plan(desc);
    // shapes, sizes and pointers this form does not take (the caller uses granq_calibrate_fakequant_fwd)
    if (!rp.ok || !fwd_cols_ok(rp.plan, desc, x, x_hat, codes_or_null) || x_hat == x) return GRANQ_ERR_UNSUPPORTED;
    if (!state || state_bytes < rp.bytes || !aligned16(state)) return GRANQ_ERR_WORKSPACE;
    ResidentArgs ra{};
    ra.x = x;
    ra.x_hat = x_hat;
    ra.codes = codes_or_null;
    ra.ch_min = ch_min;
    ra.ch_max = ch_max;
    ra.scale = scale;
    ra.zero_point = zero_point;
    ra.ws_min = (float *)state;
    ra.ws_max = (float *)((char *)state + rp.off_max);
    ra.arrive = (unsigned long long *)((char *)state + rp.off_arrive);
    ra.params = (uint64_t *)((char *)state + rp.off_params);
    ra.plan = rp.plan;
    ra.n = desc->n;
    ra.c = desc->c;
    ra.hw = desc->h * desc->w;
    ra.qmax = (float)((1 << bits) - 1);
    ra.spin_limit = spin_limit();
    hipStream_t hs = (hipStream_t)stream;
    int per_cu = 0;
    hipError_t e;
    const bool small = rp.rows_held == kResRowsSmall;
    if (desc->dtype == GRANQ_F32)
        e = small ? launch_resident<F32, kResRowsSmall>(rp.plan, ra, hs, &per_cu) : launch_resident<F32, kResRowsLarge>(rp.plan, ra, hs, &per_cu);
    else if (desc->dtype == GRANQ_BF16)
        e = small ? launch_resident<BF16, kResRowsSmall>(rp.plan, ra, hs, &per_cu) : launch_resident<BF16, kResRowsLarge>(rp.plan, ra, hs, &per_cu);
    else
        e = small ? launch_resident<F16, kResRowsSmall>(rp.plan, ra, hs, &per_cu) : launch_resident<F16, kResRowsLarge>(rp.plan, ra, hs, &per_cu);
    if (e != hipSuccess) return GRANQ_ERR_HIP;
    if (per_cu < 0) return GRANQ_ERR_UNSUPPORTED;           // the grid would not fit the chip: nothing launched
    return launched();
}

}  // extern "C"
