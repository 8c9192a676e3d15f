// Which tiling each kernel of the activation path gets for a given tensor: the tuning
// constants, the plans built from them (granq_plan.h) and the workspace layout of the
// reduction.  Host-only and free of HIP, so that the same code the library runs can be
// compiled into a host test that replays every index it produces.
#pragma once

#include <stddef.h>
#include <stdint.h>

#include "granq.h"
#include "granq_plan.h"

namespace granq {

// Vectors per lane and row for the element-wise (E: forward, backward) and the
// reduction (R) column kernels, and rows in flight per lane in the reduction.
// (Forward and backward keep GRANQ_F_ROWS / GRANQ_B_ROWS rows in flight.)
#ifndef GRANQ_E_V_F32
#define GRANQ_E_V_F32 1
#endif
#ifndef GRANQ_E_V_BF16
#define GRANQ_E_V_BF16 1
#endif
#ifndef GRANQ_R_V_F32
#define GRANQ_R_V_F32 1
#endif
#ifndef GRANQ_R_V_BF16
#define GRANQ_R_V_BF16 1
#endif
// Threads per block of the element-wise column kernels (the reduction and the
// row kernels use kBlock).
#ifndef GRANQ_E_BLOCK
#define GRANQ_E_BLOCK 64
#endif
constexpr int kEBlock = GRANQ_E_BLOCK;
// Threads per block of the reduction's first pass.
#ifndef GRANQ_R_BLOCK
#define GRANQ_R_BLOCK 256
#endif
constexpr int kRBlock = GRANQ_R_BLOCK;

// Streaming policy.  Data that cannot survive in the caches until it is needed
// again is loaded with non-temporal loads, which on MI355X stream markedly
// faster than ordinary loads; data that the next kernel re-reads is loaded
// normally so that it stays resident.
//   - a tensor of at least GRANQ_STREAM_BYTES is "large": the reduction and the
//     forward stream all of it except its last GRANQ_KEEP_BYTES, which the
//     reduction leaves in the memory-side cache and the (reverse-order) forward
//     picks up from there;
//   - the backward streams x and dy of any tensor of at least
//     GRANQ_BWD_STREAM_BYTES.
#ifndef GRANQ_STREAM_BYTES
#define GRANQ_STREAM_BYTES ((int64_t)384 << 20)
#endif
#ifndef GRANQ_KEEP_BYTES
#define GRANQ_KEEP_BYTES ((int64_t)160 << 20)
#endif
#ifndef GRANQ_BWD_STREAM_BYTES
#define GRANQ_BWD_STREAM_BYTES ((int64_t)96 << 20)
#endif

// Shape of a block of the forward that also writes gate bits: vectors per lane
// along the row and rows.  A wavefront's bits for one row are contiguous:
// 32 bytes per float32 vector slot, 64 per bfloat16 one.
// Measured on the 822 MB tensor: float32 2 x 1 costs 14 us more than the plain
// forward, 1 x 2 costs 22, 4 x 1 costs 39; bfloat16 1 x 2 and 2 x 1 cost 11-13.
#ifndef GRANQ_M_V_F32
#define GRANQ_M_V_F32 2
#endif
#ifndef GRANQ_M_ROWS_F32
#define GRANQ_M_ROWS_F32 1
#endif
#ifndef GRANQ_M_V_BF16
#define GRANQ_M_V_BF16 1
#endif
#ifndef GRANQ_M_ROWS_BF16
#define GRANQ_M_ROWS_BF16 2
#endif
inline int vec_of(granq_dtype_t dt) { return dt == GRANQ_F32 ? 4 : 8; }

inline int64_t tensor_bytes(const granq_desc_t *d) {
    return d->n * d->c * d->h * d->w * (d->dtype == GRANQ_F32 ? 4 : 2);
}

// Rows [0, nt_row_end) of a large tensor are streamed, the last GRANQ_KEEP_BYTES stay cached.
inline void split_large(ColPlan &p, const granq_desc_t *d) {
    p.nt_row_end = 0;
    if (!p.ok || tensor_bytes(d) < GRANQ_STREAM_BYTES) return;
    const int64_t row_bytes = tensor_bytes(d) / p.rows;
    const int64_t keep_rows = GRANQ_KEEP_BYTES / row_bytes;
    p.nt_row_end = p.rows > keep_rows ? p.rows - keep_rows : 0;
}

// Plans of the element-wise kernels: rows per block = rows in flight per lane.
inline ColPlan fwd_plan(const granq_desc_t *d) {
    ColPlan p = make_col_plan(d->n, d->c, d->h * d->w, vec_of(d->dtype),
                              d->dtype == GRANQ_F32 ? GRANQ_E_V_F32 : GRANQ_E_V_BF16, kEBlock,
                              (int64_t)1 << 40, GRANQ_F_ROWS);
    split_large(p, d);
    return p;
}
inline ColPlan fwd_mask_plan(const granq_desc_t *d) {
    ColPlan p = make_col_plan(d->n, d->c, d->h * d->w, vec_of(d->dtype),
                              d->dtype == GRANQ_F32 ? GRANQ_M_V_F32 : GRANQ_M_V_BF16, kEBlock,
                              (int64_t)1 << 40,
                              d->dtype == GRANQ_F32 ? GRANQ_M_ROWS_F32 : GRANQ_M_ROWS_BF16);
    split_large(p, d);
    return p;
}
inline ColPlan bwd_plan(const granq_desc_t *d) {
    ColPlan p = make_col_plan(d->n, d->c, d->h * d->w, vec_of(d->dtype),
                              d->dtype == GRANQ_F32 ? GRANQ_E_V_F32 : GRANQ_E_V_BF16, kEBlock,
                              (int64_t)1 << 40, GRANQ_B_ROWS);
    p.nt_row_end = (p.ok && tensor_bytes(d) >= GRANQ_BWD_STREAM_BYTES) ? p.rows : 0;
    return p;
}

// Plan of the reduction; it also fixes the workspace layout.  Blocks of GRANQ_R_MIN_ROWS rows
// (few partials, cheap epilogue) where that still gives the chip GRANQ_R_WANT_BLOCKS blocks
// (eight per compute unit); smaller tensors get half as many rows per block.
#ifndef GRANQ_R_WANT_BLOCKS
#define GRANQ_R_WANT_BLOCKS 2048
#endif
inline ColPlan range_plan(const granq_desc_t *d) {
    const int v = d->dtype == GRANQ_F32 ? GRANQ_R_V_F32 : GRANQ_R_V_BF16;
    ColPlan p = make_col_plan(d->n, d->c, d->h * d->w, vec_of(d->dtype), v, kRBlock,
                              GRANQ_R_TARGET_BLOCKS, GRANQ_R_MIN_ROWS);
    // (a tensor of at most 2 * GRANQ_R_MIN_ROWS rows keeps its single or two row groups: with one
    // group and whole channels per column tile the first pass is the whole reduction)
    if (p.ok && GRANQ_R_MIN_ROWS > 1 && p.rows > 2 * GRANQ_R_MIN_ROWS &&
        (int64_t)p.col_tiles * p.row_groups < GRANQ_R_WANT_BLOCKS)
        p = make_col_plan(d->n, d->c, d->h * d->w, vec_of(d->dtype), v, kRBlock,
                          GRANQ_R_TARGET_BLOCKS, (GRANQ_R_MIN_ROWS + 1) / 2);
    split_large(p, d);
    return p;
}

// Channels per column tile if the first pass alone produces final ranges (one row group, and
// no channel shared between column tiles), else 0.
inline int32_t direct_channels(const ColPlan &p) {
    if (!p.ok || p.row_groups != 1) return 0;
    if (p.col_tiles == 1) return p.channels;
    if (p.channels > 1 && p.span % p.hw == 0) return (int32_t)(p.span / p.hw);
    return 0;
}

inline size_t col_ws_floats(const ColPlan &pl) {
    return (size_t)pl.row_groups * pl.col_tiles * pl.kmax;
}

// Column path: partial minima, partial maxima, then one 8-byte hand-over slot per channel.
inline size_t col_params_offset(const ColPlan &pl) {
    return (2 * col_ws_floats(pl) * sizeof(float) + 7) & ~(size_t)7;
}
inline size_t col_ws_bytes(const ColPlan &pl) {
    return col_params_offset(pl) + (size_t)pl.channels * sizeof(uint64_t);
}

// Partials per channel: row groups x the column tiles a channel can overlap.
inline int64_t partials_per_channel(const ColPlan &pl) {
    return (int64_t)pl.row_groups * ((pl.hw - 1) / pl.span + 2);
}

// Channels per finisher block of the finishing forward, and the rows of blocks they take.
inline int64_t finisher_rows_of(const ColPlan &cp, const ColPlan &fp) {
    return ceil_div(ceil_div(cp.channels, kEBlock / 64), fp.col_tiles);
}


// ---------------------------------------------------------------------------
// The single-launch ("resident") form of ranges + parameters + forward: every block keeps its
// slice of the tensor in registers from the min / max sweep to the quantization, so the
// tensor must fit the register files of the blocks that can be on the chip together.
// ---------------------------------------------------------------------------
#ifndef GRANQ_RESIDENT_MAX_BYTES
#define GRANQ_RESIDENT_MAX_BYTES ((int64_t)64 << 20)
#endif
constexpr int kResBlock = 256;            // threads per block
constexpr int kResRowsSmall = 4;          // vectors a lane holds: 4 where that keeps the grid within
constexpr int kResRowsLarge = 16;         // the limit below, else 16
// Blocks of one launch: 256 compute units x 4 blocks of 256 threads.  The register files would
// hold twice as many of the small kind, but measured on MI355X a grid of 1600 such blocks is no
// longer on the chip all at once (the blocks that start late find the others waiting for them),
// while 1400 are; half the nominal capacity keeps a margin.
constexpr int kResBlocksSmall = 1024;
constexpr int kResBlocksLarge = 1024;

struct ResidentPlan {
    bool ok;
    int rows_held;                        // kResRowsSmall or kResRowsLarge
    ColPlan plan;                         // column tiles of kResBlock lanes x one vector, row groups of rows_held rows
    size_t off_max, off_arrive, off_params, bytes;   // state layout: partial minima at 0
};

inline ResidentPlan resident_plan(const granq_desc_t *d) {
    ResidentPlan r{};
    r.ok = false;
    if (tensor_bytes(d) > GRANQ_RESIDENT_MAX_BYTES) return r;
    ColPlan p = make_col_plan(d->n, d->c, d->h * d->w, vec_of(d->dtype), 1, kResBlock, (int64_t)1 << 40, 1);
    if (!p.ok) return r;
    for (int held : {kResRowsSmall, kResRowsLarge}) {
        const int64_t groups = ceil_div(p.rows, held);
        const int64_t limit = held == kResRowsSmall ? kResBlocksSmall : kResBlocksLarge;
        if (groups > 65535 || groups * p.col_tiles > limit) continue;
        p.rows_per_group = (int32_t)ceil_div(p.rows, groups);
        p.row_groups = (int32_t)ceil_div(p.rows, p.rows_per_group);
        r.rows_held = held;
        r.ok = true;
        break;
    }
    if (!r.ok) return r;
    p.nt_row_end = 0;
    // one wavefront gathers a channel's partials; the keys of a tile's channels sit in LDS
    if (partials_per_channel(p) > 512 || p.kmax > 4096) { r.ok = false; return r; }
    r.plan = p;
    const size_t floats = col_ws_floats(p);
    r.off_max = floats * sizeof(float);
    r.off_arrive = (2 * floats * sizeof(float) + 15) & ~(size_t)15;
    r.off_params = r.off_arrive + (size_t)p.channels * 8;
    r.bytes = r.off_params + (size_t)p.channels * 8;
    return r;
}

}  // namespace granq
