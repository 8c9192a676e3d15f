// Host replay of the index arithmetic of the activation kernels, compiled from the
// library's own planning headers (granq_plan.h, granq_tiling.h) and meant to be built with
// -fsanitize=address,undefined: for every shape on the command line (or the built-in list)
// every vector index a block of the reduction, the forward, the gate-bit forward and the
// backward would form is checked against the tensor, every partial slot against the
// workspace, and for tensors of moderate size the bytes are really touched, so that the
// sanitizer sees an access the checks missed.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <set>
#include <vector>

#include "granq_tiling.h"

using namespace granq;

static int failures = 0;
#define CHECK(cond, ...)                                            \
    do {                                                            \
        if (!(cond)) {                                              \
            if (failures < 20) { std::printf("FAIL %s:%d: ", __FILE__, __LINE__); std::printf(__VA_ARGS__); std::printf("\n"); } \
            ++failures;                                             \
        }                                                           \
    } while (0)

static const int64_t kTouchLimit = (int64_t)48 << 20;      // bytes: tensors up to here are really read

struct Tensor {
    int64_t vectors;                 // 16-byte vectors in the tensor
    std::vector<uint8_t> bytes;      // empty: too large to allocate here
    std::vector<uint8_t> seen;       // per vector: how many blocks visited it
    volatile uint8_t sink = 0;
    explicit Tensor(int64_t nbytes) : vectors(nbytes / 16) {
        if (nbytes <= kTouchLimit) {
            bytes.assign((size_t)nbytes, 1);
            seen.assign((size_t)vectors, 0);
        }
    }
    void visit(int64_t idx, const char *who) {
        CHECK(idx >= 0 && idx < vectors, "%s: vector %lld outside [0, %lld)", who, (long long)idx, (long long)vectors);
        if (!bytes.empty() && idx >= 0) {
            sink = bytes[(size_t)idx * 16] + bytes[(size_t)idx * 16 + 15];      // the sanitizer's check
            if (idx < vectors) ++seen[(size_t)idx];
        }
    }
    void exactly_once(const char *who) {
        for (size_t i = 0; i < seen.size(); ++i)
            if (seen[i] != 1) { CHECK(false, "%s: vector %zu visited %d times", who, i, (int)seen[i]); break; }
        std::fill(seen.begin(), seen.end(), 0);
    }
};

template <int MODE, int VEC>
static void lane_channels(uint32_t tcol, const ColPlan &pl, std::vector<int32_t> &out) {
    constexpr int NS = Slots<MODE, VEC>::N;
    int32_t ch[NS];
    const uint32_t split = vector_channels<MODE, VEC, NS>(tcol, pl, ch);
    out.clear();
    for (int e = 0; e < VEC; ++e) {
        int32_t c = MODE == kOne ? ch[0] : (MODE == kEach ? ch[e < NS ? e : 0] : ((uint32_t)e < split ? ch[0] : ch[NS > 1 ? 1 : 0]));
        out.push_back(c);
    }
}

template <int VEC>
static void channels_of(uint32_t tcol, const ColPlan &pl, std::vector<int32_t> &out) {
    if (pl.mode == kOne) lane_channels<kOne, VEC>(tcol, pl, out);
    else if (pl.mode == kTwo) lane_channels<kTwo, VEC>(tcol, pl, out);
    else lane_channels<kEach, VEC>(tcol, pl, out);
}

// A column kernel's walk: grid (col_tiles, row_groups), `block` threads, v vectors per lane.
template <int VEC>
static void walk(const ColPlan &pl, int block, int v_per_lane, Tensor &t, const granq_desc_t &d, const char *who,
                 bool check_channels) {
    CHECK(pl.rows * pl.row_len * (int64_t)(16 / VEC) == t.vectors * 16, "%s: rows x row_len is not the tensor", who);
    CHECK(pl.row_groups >= 1 && pl.row_groups <= 65535, "%s: %d row groups", who, pl.row_groups);
    CHECK((int64_t)(pl.row_groups - 1) * pl.rows_per_group < pl.rows &&
          pl.rows <= (int64_t)pl.row_groups * pl.rows_per_group, "%s: row groups do not tile the rows", who);
    CHECK(pl.span == block * VEC * v_per_lane, "%s: span %d", who, pl.span);
    const int64_t row_vecs = pl.row_len / VEC;
    const int64_t true_len = pl.row_len / pl.fold;
    const int64_t hw = d.c == 1 ? true_len : d.h * d.w;
    std::vector<int32_t> chans;
    for (int64_t j = 0; j < pl.col_tiles; ++j) {
        const int32_t ch_first = (int32_t)fastdiv((uint32_t)(j * pl.span), pl.hw_div);
        for (int lane = 0; lane < block; ++lane)
            for (int v = 0; v < v_per_lane; ++v) {
                const uint32_t col = (uint32_t)(j * pl.span) + (uint32_t)(lane + v * block) * VEC;
                if (col >= (uint32_t)pl.row_len) continue;
                const uint32_t cv = col / VEC;
                if (check_channels) {
                    const uint32_t tcol = true_column(col, pl);
                    channels_of<VEC>(tcol, pl, chans);
                    for (int e = 0; e < VEC; ++e) {
                        const int64_t want = ((int64_t)(col + e) % true_len) / hw;
                        CHECK(chans[e] == want, "%s: column %u element %d: channel %d, expected %lld", who, col, e,
                              chans[e], (long long)want);
                        const int32_t k = chans[e] - ch_first;
                        CHECK(k >= 0 && k < pl.kmax, "%s: tile %lld: channel slot %d outside [0, %d)", who, (long long)j, k, pl.kmax);
                    }
                }
                // rows: all of them where the tensor is touched for real, else the ends of every group
                if (!t.bytes.empty()) {
                    for (int64_t r = 0; r < pl.rows; ++r) t.visit(r * row_vecs + cv, who);
                } else {
                    for (int64_t p = 0; p < pl.row_groups; p += (pl.row_groups > 64 ? pl.row_groups - 1 : 1)) {
                        const int64_t r0 = p * pl.rows_per_group;
                        const int64_t r1 = r0 + pl.rows_per_group < pl.rows ? r0 + pl.rows_per_group : pl.rows;
                        t.visit(r0 * row_vecs + cv, who);
                        t.visit((r1 - 1) * row_vecs + cv, who);
                    }
                }
            }
    }
    if (!t.bytes.empty()) t.exactly_once(who);
}

template <int VEC>
static void check_shape(const granq_desc_t &d) {
    const int esize = 16 / VEC;
    const int64_t e = d.n * d.c * d.h * d.w;
    const ColPlan rp = range_plan(&d), fp = fwd_plan(&d), mp = fwd_mask_plan(&d), bp = bwd_plan(&d);
    if (!rp.ok) {
        CHECK(!fp.ok && !bp.ok, "plans disagree on eligibility");
        CHECK((d.c * d.h * d.w) % VEC != 0 || (d.c == 1 && e % VEC != 0), "an eligible shape was refused");
        return;
    }
    CHECK(fp.ok && mp.ok && bp.ok, "plans disagree on eligibility");
    Tensor t(e * esize);
    const int rv = d.dtype == GRANQ_F32 ? GRANQ_R_V_F32 : GRANQ_R_V_BF16;
    const int ev = d.dtype == GRANQ_F32 ? GRANQ_E_V_F32 : GRANQ_E_V_BF16;
    const int mv = d.dtype == GRANQ_F32 ? GRANQ_M_V_F32 : GRANQ_M_V_BF16;
    walk<VEC>(rp, kRBlock, rv, t, d, "reduction", true);
    walk<VEC>(fp, kEBlock, ev, t, d, "forward", true);
    walk<VEC>(mp, kEBlock, mv, t, d, "gate-bit forward", true);
    walk<VEC>(bp, kEBlock, ev, t, d, "backward", true);

    // workspace: partials, then the hand-over slots
    const size_t floats = col_ws_floats(rp);
    CHECK(col_params_offset(rp) >= 2 * floats * sizeof(float) && col_params_offset(rp) % 8 == 0, "hand-over slots misplaced");
    CHECK(col_ws_bytes(rp) == col_params_offset(rp) + (size_t)rp.channels * 8, "workspace size");
    size_t need = 0;
    // (granq_workspace_bytes itself lives in the library; its column part is col_ws_bytes)
    need = col_ws_bytes(rp);
    CHECK(need < ((size_t)1 << 40), "workspace absurd");
    // every (block, slot) the first pass writes lies in the workspace, and the gather of every
    // channel reads exactly the slots that can hold that channel's data
    CHECK(partial_slot(rp, rp.row_groups - 1, rp.col_tiles - 1, rp.kmax - 1) == (int64_t)floats - 1, "last partial slot");
    const int64_t true_len = rp.row_len / rp.fold;
    const int64_t hw = rp.hw;
    const int64_t channels = rp.channels;
    CHECK(channels == (d.c == 1 ? 1 : d.c), "channel count %lld", (long long)channels);
    std::vector<std::set<int64_t>> holds((size_t)channels);      // tiles whose columns hold data of channel c
    for (int64_t j = 0; j < rp.col_tiles; ++j) {
        const int64_t c0 = j * rp.span;
        const int64_t c1 = (c0 + rp.span < rp.row_len ? c0 + rp.span : rp.row_len) - 1;
        if (rp.fold > 1) { for (int64_t c = 0; c < channels; ++c) holds[(size_t)c].insert(j); continue; }
        for (int64_t c = (c0 % true_len) / hw; c <= (c1 % true_len) / hw; ++c) holds[(size_t)c].insert(j);
    }
    for (int64_t c = 0; c < channels; ++c) {
        const ChannelPartials cp = channel_partials(rp, c);
        CHECK(cp.total == cp.nj * (uint32_t)rp.row_groups && cp.total >= 1, "channel %lld: %u partials", (long long)c, cp.total);
        CHECK((int64_t)cp.total <= partials_per_channel(rp), "channel %lld: more partials than the bound", (long long)c);
        std::set<int64_t> tiles;
        for (uint32_t i = 0; i < cp.total; i += (cp.total > 4096 ? cp.total / 64 : 1)) {
            const int64_t at = channel_partial_slot(rp, c, cp, i);
            CHECK(at >= 0 && at < (int64_t)floats, "channel %lld item %u: slot %lld outside the workspace", (long long)c, i, (long long)at);
            const int64_t jj = (at / rp.kmax) % rp.col_tiles, k = at % rp.kmax;
            CHECK((jj * rp.span) / hw + k == c, "channel %lld item %u reads a slot of channel %lld", (long long)c, i,
                  (long long)((jj * rp.span) / hw + k));
            tiles.insert(jj);
        }
        if (cp.total <= 4096)
            for (int64_t j : holds[(size_t)c]) CHECK(tiles.count(j) == 1, "channel %lld: tile %lld is never gathered", (long long)c, (long long)j);
    }
    // single-pass reduction only where a block holds whole channels
    const int32_t direct = direct_channels(rp);
    if (direct > 0) {
        CHECK(rp.row_groups == 1, "single-pass reduction with %d row groups", rp.row_groups);
        for (int64_t c = 0; c < channels; ++c) CHECK(holds[(size_t)c].size() == 1, "single pass, but channel %lld spans tiles", (long long)c);
        CHECK(direct <= rp.kmax, "single pass writes %d channels per tile, %d slots exist", direct, rp.kmax);
    }
    // the finishing forward's grid
    const int64_t fin = finisher_rows_of(rp, fp);
    CHECK(fin * fp.col_tiles * (kEBlock / 64) >= channels, "finisher rows do not cover the channels");

    // the single-launch form: its walk, its state layout, and its arrival counts -- a channel
    // completes when exactly channel_partials().total blocks have counted themselves in, and a block
    // counts itself in at the channels first .. last of its tile
    const ResidentPlan res = resident_plan(&d);
    if (res.ok) {
        const ColPlan &qp = res.plan;
        CHECK(qp.rows_per_group <= res.rows_held, "a block holds %d rows, its lanes %d", qp.rows_per_group, res.rows_held);
        CHECK((int64_t)qp.col_tiles * qp.row_groups <= (res.rows_held == kResRowsSmall ? kResBlocksSmall : kResBlocksLarge),
              "resident grid of %lld blocks", (long long)qp.col_tiles * qp.row_groups);
        walk<VEC>(qp, kResBlock, 1, t, d, "resident forward", true);
        const size_t qfloats = col_ws_floats(qp);
        CHECK(res.off_max == qfloats * 4 && res.off_arrive >= 2 * qfloats * 4 && res.off_arrive % 8 == 0 &&
              res.off_params == res.off_arrive + (size_t)qp.channels * 8 && res.bytes == res.off_params + (size_t)qp.channels * 8,
              "resident state layout");
        std::vector<int64_t> arrivals((size_t)qp.channels, 0);
        for (int64_t j = 0; j < qp.col_tiles; ++j) {
            const int64_t first = fastdiv((uint32_t)(j * qp.span), qp.hw_div);
            const int64_t end = (j + 1) * qp.span < qp.row_len ? (j + 1) * qp.span : qp.row_len;
            int64_t last = fastdiv((uint32_t)(end - 1), qp.hw_div);
            if (last > qp.channels - 1) last = qp.channels - 1;
            CHECK(last - first < qp.kmax, "tile %lld arrives at %lld channels, %d slots", (long long)j, (long long)(last - first + 1), qp.kmax);
            for (int64_t c = first; c <= last; ++c) arrivals[(size_t)c] += qp.row_groups;
        }
        for (int64_t c = 0; c < qp.channels; ++c)
            CHECK(arrivals[(size_t)c] == (int64_t)channel_partials(qp, c).total,
                  "channel %lld: %lld blocks arrive, %u are expected", (long long)c, (long long)arrivals[(size_t)c],
                  channel_partials(qp, c).total);
    } else {
        CHECK(e * esize > GRANQ_RESIDENT_MAX_BYTES || rp.rows > 0, "resident plan refused");
    }
}

int main(int argc, char **argv) {
    static const int64_t shapes[][4] = {
        // small shapes of the parity tests
        {8, 16, 32, 32}, {5, 37, 9, 8}, {6, 100, 7, 7}, {3, 40, 1, 1}, {9, 24, 14, 14}, {4, 3000, 1, 1},
        {1, 1, 1, 16384}, {2, 1, 5, 4}, {1, 64, 1, 1152}, {7, 12, 14, 14}, {1, 2048, 7, 7}, {13, 8, 7, 7},
        {17, 520, 2, 2}, {4, 4, 64, 65}, {1, 1, 1, 4}, {1, 4, 1, 1}, {31, 8, 1, 3}, {200001, 4, 1, 4}, {70001, 3, 2, 2},
        {2, 3, 7, 7}, {5, 7, 3, 3}, {1, 1, 1, 5}, {3, 1, 7, 3}, {1, 1, 1, 1}, {2, 5, 1, 1}, {4, 9, 5, 5},
        {64, 24, 28, 28}, {700, 100, 7, 7}, {40000, 40, 1, 1}, {300, 3, 40, 40}, {512, 64, 1, 1}, {489, 10, 2, 2},
        // the five workloads at batch 256 (batch 8 for the first)
        {256, 16, 32, 32}, {256, 32, 16, 16}, {256, 64, 8, 8},
        {256, 64, 112, 112}, {256, 64, 56, 56}, {256, 128, 28, 28}, {256, 256, 14, 14}, {256, 512, 7, 7},
        {256, 32, 112, 112}, {256, 96, 112, 112}, {256, 96, 56, 56}, {256, 144, 56, 56}, {256, 144, 28, 28},
        {256, 192, 28, 28}, {256, 192, 14, 14}, {256, 384, 14, 14}, {256, 576, 14, 14}, {256, 576, 7, 7},
        {256, 960, 7, 7}, {256, 16, 112, 112}, {256, 24, 56, 56}, {256, 32, 28, 28}, {256, 64, 14, 14},
        {256, 96, 14, 14}, {256, 160, 7, 7}, {256, 320, 7, 7},
        {256, 256, 56, 56}, {256, 128, 56, 56}, {256, 512, 28, 28}, {256, 1024, 14, 14}, {256, 512, 14, 14},
        {256, 2048, 7, 7}, {256, 1024, 7, 7},
        // views
        {1, 1, 1, 205520896}, {1, 65536, 7, 7}, {802816, 64, 1, 1},
    };
    int count = 0;
    for (const auto &sh : shapes)
        for (int dt = 0; dt < 2; ++dt) {
            granq_desc_t d{sh[0], sh[1], sh[2], sh[3], dt == 0 ? GRANQ_F32 : GRANQ_BF16};
            const int before = failures;
            if (dt == 0) check_shape<4>(d); else check_shape<8>(d);
            if (failures != before)
                std::printf("  ^ shape {%lld,%lld,%lld,%lld} %s\n", (long long)sh[0], (long long)sh[1], (long long)sh[2],
                            (long long)sh[3], dt == 0 ? "float32" : "16-bit");
            ++count;
        }
    std::printf("%d shape/type pairs replayed, %d failures\n", count, failures);
    return failures ? 1 : 0;
    (void)argc; (void)argv;
}
