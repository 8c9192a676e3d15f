// Host-side launch planning for the GranQ kernels.
//
// A dense NCHW tensor is a matrix of N rows by L = C*H*W columns, and the
// channel of an element depends on its COLUMN only: channel = column / (H*W).
// The vectorised kernels exploit this: a block owns a span of columns and walks
// down the rows, so every lane works for the same channel(s) during its whole
// life and keeps their scale / zero-point (or its running min / max) in
// registers.  No index arithmetic and no table lookup is left in the loop over
// the data.
//
//   columns:  J tiles of `span` = kBlock * VEC * V elements (VEC = 16 bytes'
//             worth of elements, V vectors per lane and row)
//   rows:     P groups of `rows_per_group` consecutive rows
//   grid:     (J, P) blocks, column tile fastest, so that blocks that are
//             resident together read neighbouring spans of the same rows.
//
// A tensor with a single channel (the layer-wise view {1,1,1,E}) has only one
// row; since every element then belongs to channel 0 the matrix may be folded
// to any rows x columns factorisation, and the plan does so.
//
// Short rows (a channels-last tensor seen as {N*H*W, C, 1, 1} has rows of C
// elements) would leave most lanes of a block without a column.  The plans
// therefore glue `fold` consecutive rows into one row of the matrix they walk:
// a lane's column, taken modulo the true row length, still fixes its channel(s)
// for good.  The fold is chosen so that the glued row is exactly what one block
// spans or less, and divides the row count.
#pragma once

#include <stdint.h>
#include <stddef.h>

namespace granq {

// Tuning (defaults from sweeps on MI355X; -D overrides).
// Element-wise kernels (forward, backward) run best as very many short blocks:
// a block that issues all its loads at once and retires keeps the memory system
// busier than long-lived blocks marching in lockstep.  A block of the forward
// handles GRANQ_F_ROWS rows of its column tile, one of the backward
// GRANQ_B_ROWS.  The reduction prefers fatter blocks (fewer partials, cheaper
// epilogue): at least GRANQ_R_MIN_ROWS rows per block.
#ifndef GRANQ_F_ROWS
#define GRANQ_F_ROWS 2
#endif
#ifndef GRANQ_B_ROWS
#define GRANQ_B_ROWS 1
#endif
#ifndef GRANQ_R_TARGET_BLOCKS
#define GRANQ_R_TARGET_BLOCKS 1000000
#endif
#ifndef GRANQ_R_MIN_ROWS
#define GRANQ_R_MIN_ROWS 8
#endif
// Blocks the fallback (row) kernels aim for: 256 compute units x 8 blocks.
#ifndef GRANQ_ROW_TARGET_BLOCKS
#define GRANQ_ROW_TARGET_BLOCKS 2048
#endif

#if defined(__HIPCC__)
#define GRANQ_PLAN_HD __host__ __device__
#else
#define GRANQ_PLAN_HD
#endif

// Division of a 32-bit unsigned number by a constant chosen at run time
// (Granlund & Montgomery, "Division by invariant integers using
// multiplication", 1994): with l = ceil(log2 d) and
// m = floor(2^32 * (2^l - d) / d) + 1,
//     n / d = (t + ((n - t) >> min(l,1))) >> max(l-1,0),   t = mulhi(m, n),
// exact for every 32-bit n.  Five integer instructions instead of the ~30 of a
// general division.
struct FastDiv {
    uint32_t d, m, s1, s2;
};

inline FastDiv make_fastdiv(uint32_t d) {
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    uint64_t m = (((uint64_t)1 << 32) * (((uint64_t)1 << l) - d)) / d + 1;
    FastDiv f;
    f.d = d;
    f.m = (uint32_t)m;
    f.s1 = l < 1 ? l : 1;
    f.s2 = l > 0 ? l - 1 : 0;
    return f;
}

GRANQ_PLAN_HD inline uint32_t fastdiv(uint32_t n, const FastDiv &f) {
    uint32_t t = (uint32_t)(((uint64_t)f.m * n) >> 32);
    return (t + ((n - t) >> f.s1)) >> f.s2;
}

struct ColPlan {
    int64_t rows;            // rows of the (possibly folded) matrix
    int64_t row_len;         // columns (elements per row)
    int64_t hw;              // elements per channel within a row
    int32_t channels;        // channels per row
    int32_t span;            // columns per block
    int32_t col_tiles;       // J
    int32_t row_groups;      // P
    int32_t rows_per_group;
    int32_t kmax;            // most channels any column tile touches
    int64_t nt_row_end;      // rows below this are loaded non-temporally (streamed)
    FastDiv hw_div;          // column -> channel
    bool uniform;            // every 16-byte vector lies inside one channel
    int32_t mode;            // 0: one channel per vector, 1: at most two, 2: up to one per element
    int32_t fold;            // true rows glued into one row of this matrix (1: none)
    bool v_same;             // glued rows: a lane's V vectors all see the same channels
    FastDiv true_len_div;    // column -> column within the true row (used when fold > 1)
    bool ok;                 // false: shape not eligible for the vector kernels
};

// Column within the true row of the tensor.
GRANQ_PLAN_HD inline uint32_t true_column(uint32_t col, const ColPlan &p) {
    if (p.fold <= 1) return col;
    return col - fastdiv(col, p.true_len_div) * p.true_len_div.d;
}

// How the elements of one 16-byte vector map to channels (template parameter MODE):
//   kOne   H*W is a multiple of the vector width: the whole vector is one channel
//   kTwo   H*W >= vector width: at most two channels, elements [0, split) and [split, VEC)
//   kEach  H*W < vector width: every element may have its own channel
constexpr int kOne = 0, kTwo = 1, kEach = 2;
template <int MODE, int VEC>
struct Slots { static constexpr int N = MODE == kOne ? 1 : (MODE == kTwo ? 2 : VEC); };

// Channels of this lane's vector starting at column `col`: ch[] per slot, and the
// number of leading elements that belong to the first channel.
template <int MODE, int VEC, int NS>
GRANQ_PLAN_HD inline uint32_t vector_channels(uint32_t col, const ColPlan &plan, int32_t (&ch)[NS]) {
    const uint32_t c0 = fastdiv(col, plan.hw_div);
    const uint32_t rem = col - c0 * plan.hw_div.d;
    if (MODE == kEach) {
        uint32_t c = c0, r = rem;
        ch[0] = (int32_t)c;
        for (int e = 1; e < NS; ++e) {
            r += 1;
            if (r == plan.hw_div.d) { r = 0; c += 1; }
            ch[e] = (int32_t)c;
        }
        return VEC;
    }
    ch[0] = (int32_t)c0;
    if (MODE == kOne) return VEC;
    const uint32_t left = plan.hw_div.d - rem;           // elements of channel c0 from col on
    const uint32_t split = left < (uint32_t)VEC ? left : (uint32_t)VEC;
    ch[NS > 1 ? 1 : 0] = (int32_t)(split < (uint32_t)VEC ? c0 + 1 : c0);
    return split;
}


// The first pass of the reduction leaves one partial min / max per (row group p, column tile
// j, channel slot k), k = channel - first channel of tile j, at this index of the workspace.
GRANQ_PLAN_HD inline int64_t partial_slot(const ColPlan &plan, int64_t p, int64_t j, int64_t k) {
    return (p * plan.col_tiles + j) * plan.kmax + k;
}

// The partials of channel c: those of all row groups and of the column tiles j_lo .. j_lo + nj - 1
// that overlap the channel, `total` in all; item i of them sits at channel_partial_slot().
struct ChannelPartials {
    uint32_t j_lo, nj, total;                  // total < 2^31: tiles x 65535 row groups at most
};
GRANQ_PLAN_HD inline ChannelPartials channel_partials(const ColPlan &plan, int64_t c) {
    ChannelPartials cp;
    cp.j_lo = (uint32_t)((c * plan.hw) / plan.span);
    const uint32_t j_hi = (uint32_t)(((c + 1) * plan.hw - 1) / plan.span);
    cp.nj = j_hi - cp.j_lo + 1;
    cp.total = cp.nj * (uint32_t)plan.row_groups;
    return cp;
}
GRANQ_PLAN_HD inline int64_t channel_partial_slot(const ColPlan &plan, int64_t c, const ChannelPartials &cp,
                                                  uint32_t i) {
    const uint32_t pp = i / cp.nj;
    const uint32_t jj = cp.j_lo + (i - pp * cp.nj);
    const int64_t k = c - ((int64_t)jj * plan.span) / plan.hw;
    return partial_slot(plan, pp, jj, k);
}

inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// vec = elements per 16 bytes, v = vectors per lane and row, block = threads.
inline ColPlan make_col_plan(int64_t n, int64_t c, int64_t hw, int vec, int v, int block,
                             int64_t target_blocks, int64_t min_rows) {
    ColPlan p{};
    p.ok = false;
    p.fold = 1;
    p.v_same = false;
    int64_t rows = n, row_len = c * hw, chan = c, per = hw;
    if (c == 1) {
        // fold rows * row_len = E so that rows is a power of two up to 1024
        // and the row length stays a multiple of the vector width
        int64_t e = n * hw;
        if (e % vec != 0) return p;
        int64_t r = 1;
        while (r < 1024 && (e / vec) % (2 * r) == 0 && e / (2 * r) >= (int64_t)block * vec * v) r *= 2;
        rows = r;
        row_len = e / r;
        per = row_len;
        chan = 1;
    }
    if (row_len % vec != 0) return p;
    if (row_len >= (int64_t)1 << 31) return p;
    p.true_len_div = make_fastdiv((uint32_t)row_len);
    const int64_t block_span = (int64_t)block * vec * v;
    if (c > 1 && row_len < block_span) {
        // the largest fold that keeps the glued row within one block's span and divides the rows
        int64_t f = block_span / row_len;
        while (f > 1 && rows % f != 0) --f;
        p.fold = (int32_t)f;
        // a lane's vectors are block * vec columns apart: a whole number of true rows?
        p.v_same = f > 1 && ((int64_t)block * vec) % row_len == 0;
        rows /= f;
        row_len *= f;
    }
    p.rows = rows;
    p.row_len = row_len;
    p.hw = per;
    p.channels = (int32_t)chan;
    p.span = block * vec * v;
    p.col_tiles = (int32_t)ceil_div(row_len, p.span);
    int64_t want = ceil_div(target_blocks, p.col_tiles);
    int64_t most = rows / min_rows > 0 ? rows / min_rows : 1;
    int64_t groups = want < most ? want : most;
    if (groups < 1) groups = 1;
    if (groups > 65535) groups = 65535;              // row groups ride on gridDim.y
    p.rows_per_group = (int32_t)ceil_div(rows, groups);
    p.row_groups = (int32_t)ceil_div(rows, p.rows_per_group);
    p.hw_div = make_fastdiv((uint32_t)per);
    int64_t k = (p.span - 1) / per + 2;
    p.kmax = (int32_t)(k < chan ? k : chan);
    p.uniform = (per % vec) == 0;
    p.mode = p.uniform ? 0 : (per >= vec ? 1 : 2);
    p.ok = true;
    return p;
}

// Fallback ("row") plan: one channel per block, P groups of rows; where the rows alone do not
// give a channel its share of blocks (few samples, long slabs: the layer-wise view is one
// slab), every slab of H*W elements is also cut into `chunks` pieces of `chunk_len` elements.
struct RowPlan {
    int32_t row_groups;
    int32_t rows_per_group;
    int32_t chunks;
    int64_t chunk_len;
};

inline RowPlan make_row_plan(int64_t n, int64_t c, int64_t hw) {
    RowPlan p{};
    int64_t want = ceil_div(GRANQ_ROW_TARGET_BLOCKS, c);
    // keep at least ~4096 elements per block where the tensor allows it
    int64_t min_rows = ceil_div(4096, hw);
    int64_t most = n / min_rows > 0 ? n / min_rows : 1;
    int64_t groups = want < most ? want : most;
    if (groups < 1) groups = 1;
    p.rows_per_group = (int32_t)ceil_div(n, groups);
    p.row_groups = (int32_t)ceil_div(n, p.rows_per_group);
    int64_t chunks = ceil_div(want, p.row_groups);
    const int64_t most_chunks = hw / 4096 > 0 ? hw / 4096 : 1;
    if (chunks > most_chunks) chunks = most_chunks;
    if (chunks > 32768) chunks = 32768;
    p.chunk_len = ceil_div(hw, chunks);
    p.chunks = (int32_t)ceil_div(hw, p.chunk_len);
    return p;
}

}  // namespace granq
