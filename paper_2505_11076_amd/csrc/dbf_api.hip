// C ABI of libdbf: argument checks, the layer / stack objects and kernel dispatch.
// Every operation of the layer product itself runs in the HIP kernels; this file only
// validates, allocates at pack time, and launches.
#include <algorithm>
#include <climits>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "dbf_kernels.h"

namespace {

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline bool shape_ok(int n_in, int n_out, int k) {
    return n_in >= 1 && n_out >= 1 && k >= 1 && n_in <= DBF_MAX_DIM && n_out <= DBF_MAX_DIM &&
           k <= DBF_MAX_DIM;
}

#define DBF_HIP_TRY(expr)                  \
    do {                                   \
        if ((expr) != hipSuccess) {        \
            (void)hipGetLastError();       \
            return DBF_EHIP;               \
        }                                  \
    } while (0)

// Matrix-core items of one stage of one layer.  The number of row tiles per item follows
// `pattern`, cyclically; `phase` carries the position in the pattern from layer to layer.
void append_items(std::vector<DbfItem>& out, const DbfStage& st, int layer, bool stage_a,
                  int need, const std::vector<int>& pattern, int* phase) {
    for (int rt = 0; rt < st.n_rt;) {
        const int span = pattern[(size_t)(*phase)++ % pattern.size()];
        DbfItem it;
        std::memset(&it, 0, sizeof(it));
        it.bits = st.bits + (size_t)rt * st.n_ct * DBF_TILE_BYTES;
        it.in_scale = st.in_scale;
        it.row_scale = st.row_scale + (size_t)rt * DBF_TILE_ROWS;
        it.t = st.t;
        it.io_off = stage_a ? st.y_off : st.x_off;
        it.n_ct = st.n_ct;
        it.nrt = (st.n_rt - rt < span) ? (st.n_rt - rt) : span;
        it.row0 = rt * DBF_TILE_ROWS;
        it.rows = st.rows;
        it.cols = st.cols;
        it.t_stride = st.t_stride;
        it.layer = layer;
        it.need = need;
        it.stage_a = stage_a ? 1 : 0;
        it.ct0 = 0;
        it.ct_n = st.n_ct;
        it.pieces = 1;
        it.q_in = st.q_in;
        out.push_back(it);
        rt += it.nrt;
    }
}

// Tuning and test hooks (include/dbf.h, "tuning and test hooks"): default, smallest and largest value per knob.
struct Knob {
    int value, def, lo, hi;
};
Knob g_knobs[DBF_TUNE_COUNT_] = {
    {-1, -1, -1, 64},             // DBF_TUNE_COL_PIECES
    {0, 0, 0, 65536},             // DBF_TUNE_PIECE_TARGET
    {24, 24, 1, 4096},            // DBF_TUNE_PIECE_MIN_TILES
    {64, 64, 0, 65536},           // DBF_TUNE_PIECE_NEVER_TILES
    {768, 768, 0, 1 << 20},       // DBF_TUNE_PIECE_MAX_ROW_TILES
    {0, 0, 0, DBF_MAX_SPAN},      // DBF_TUNE_STACK_SPAN_B
    {0, 0, 0, DBF_MAX_SPAN},      // DBF_TUNE_STACK_SPAN_A
    {-1, -1, -1, 3},              // DBF_TUNE_SHARED_Q
    {2, 2, 1, DBF_MAX_BATCH + 1}, // DBF_TUNE_SHARED_MIN_BATCH
    {52, 52, 16, 64},             // DBF_TUNE_SHARED_LDS_KB
    {250000, 250000, 0, 10000000},// DBF_TUNE_WAIT_LIMIT_US
    {-1, -1, -1, 1},              // DBF_TUNE_LONG_ROWS
    {-1, -1, -1, 1024},           // DBF_TUNE_GEMM_SPLITS
    {1024, 1024, 0, 1 << 20},     // DBF_TUNE_FUSED_MIN_B_ITEMS
    {256, 256, 0, 1 << 20},       // DBF_TUNE_WIDE_WG_MAX_ITEMS
    {256, 256, 0, 1 << 20},       // DBF_TUNE_FP4_MAX_ITEMS
};

// Column pieces.  Cutting pays only for long rows: every piece pays the workgroup's prologue (it reads
// the whole input row for the quantisation scale) and the last piece an extra epilogue, which at 4096
// columns costs more than the added parallelism gains (measured 17 vs 14 us for a 4096 x 4096 layer
// alone).  So rows of up to DBF_TUNE_PIECE_NEVER_TILES column tiles are never cut, pieces hold at least
// DBF_TUNE_PIECE_MIN_TILES tiles, and a stage is cut until it offers about PIECE_TARGET_ITEMS workgroups.
constexpr int PIECE_TARGET_ITEMS = 256;
constexpr int PIECE_TARGET_STREAM = 1024;  // the same for launches that hold more row tiles than that already

// Pieces per row tile of a stage with n_ct column tiles when the launch holds stage_row_tiles row
// tiles of that stage.
int pieces_for(int n_ct, int stage_row_tiles) {
    const int forced = dbf_tune(DBF_TUNE_COL_PIECES);
    if (forced == 0) return 1;
    const int min_tiles = dbf_tune(DBF_TUNE_PIECE_MIN_TILES);
    if (forced < 0 && n_ct <= dbf_tune(DBF_TUNE_PIECE_NEVER_TILES)) return 1;
    // (a stage of several layers with a few hundred long row tiles wants two rounds of items, not a quarter of one:
    //  8192 x 28672 streams of 8-13 layers gained 4-19 % with their rows cut in two, one layer alone lost with more
    //  than about 256 items)
    int target = dbf_tune(DBF_TUNE_PIECE_TARGET);
    if (target == 0) target = stage_row_tiles > PIECE_TARGET_ITEMS ? PIECE_TARGET_STREAM : PIECE_TARGET_ITEMS;
    int want = forced > 0 ? forced : (target + stage_row_tiles - 1) / stage_row_tiles;
    const int fit = n_ct / (forced > 0 ? 8 : min_tiles);
    if (want > fit) want = fit;
    return want < 1 ? 1 : want;
}

// Items of one stage of one layer with every row tile cut into `pieces` column pieces of (almost)
// equal size.  acc / cnt: this stage's accumulators (row 0) and arrival counters (row tile 0).
void append_piece_items(std::vector<DbfItem>& out, const DbfStage& st, int layer, bool stage_a, int need,
                        int pieces, int* acc, int acc_stride, int* cnt) {
    for (int rt = 0; rt < st.n_rt; ++rt) {
        for (int pc = 0; pc < pieces; ++pc) {
            DbfItem it;
            std::memset(&it, 0, sizeof(it));
            it.bits = st.bits + (size_t)rt * st.n_ct * DBF_TILE_BYTES;
            it.in_scale = st.in_scale;
            it.row_scale = st.row_scale + (size_t)rt * DBF_TILE_ROWS;
            it.t = st.t;
            it.io_off = stage_a ? st.y_off : st.x_off;
            it.n_ct = st.n_ct;
            it.nrt = 1;
            it.row0 = rt * DBF_TILE_ROWS;
            it.rows = st.rows;
            it.cols = st.cols;
            it.t_stride = st.t_stride;
            it.layer = layer;
            it.need = need;
            it.stage_a = stage_a ? 1 : 0;
            it.ct0 = (int)((long long)st.n_ct * pc / pieces);
            it.ct_n = (int)((long long)st.n_ct * (pc + 1) / pieces) - it.ct0;
            it.pieces = pieces;
            it.acc_stride = acc_stride;
            it.acc = acc + (size_t)rt * DBF_TILE_ROWS;
            it.cnt = cnt + (size_t)rt * DBF_PIECE_CNT_STRIDE;
            it.q_in = st.q_in;
            out.push_back(it);
        }
    }
}

// Row tiles per workgroup for one stage of one layer in a launch whose stage holds `stage_tiles` tiles
// (1 KiB each) in all.  The input row is quantised once per workgroup, so longer items amortise that
// prologue; shorter ones leave more items to balance the end of the launch.  Measured on streams of
// 0.25-1 GB of signs: items of 128-256 KiB with about 2000 of them per stage do best (4096 x 4096 layers,
// k = 2048: 5.7 TB/s at 2 and 4 row tiles for the two stages against 5.4 at 1 and 1; k = 4096: 5.7 TB/s at
// 2 and 2 against 4.8 at 4 and 4), and rows too wide for the one-pass prologue, which read the input twice,
// always want the longest items (8192 x 8192, k = 8192: 3.9 TB/s at 4 against 3.0 at 1).
// Long-rows plans take this list at batch 1, where their workgroups read the quantised input tile by tile and
// have no prologue to amortise: they did best with about 1000 items per stage (8192 x 28672 streams, k = 6371:
// 4.7 TB/s at 1 and 2 row tiles per item against 3.9 at 4, which makes 240 items).
// Items are at most 256 KiB and at most 8 row tiles (rows of 32-48 column tiles get 8 and 5 instead of 4: the 224-layer
// Llama-2-7B stack 5.92 -> 6.01 TB/s, nothing else moved by more than 1 %), and a layer's items are of equal length
// to within one row tile (balanced_spans).  Asking for half as many items of twice the size helped where it left
// whole rounds of equal items (512 layers of 4096 x 4096, k = 2048: +2.3 %; 64 of them: +7 %) and cost 2.5-7 % on
// streams of k = 3072-4096 and of 8192 x 8192 layers: not taken.
int auto_span(const DbfStage& st, long long stage_tiles, bool long_rows, bool uniform) {
    // (a stage large enough for a thousand items of 512 KiB gets those: one long item per workgroup slot of the chip instead
    //  of two rounds of 256 KiB -- since an item stores its rows once, at its end, its head and tail weigh more than an
    //  uneven last round.  512 / 1024 layers of 4096 x 4096, k = 2048, same box: 6.11 -> 6.23-6.29 / 6.24 -> 6.28-6.31 TB/s.
    //  Eight row tiles forced on smaller launches lose, by up to half on wide rows; and only where all layers have one shape:
    //  the 224 mixed layers of a 7B decoder at 1.5 bits fell from 6.2 to 5.4 TB/s with it -- one round of items of very
    //  different lengths.)
    const bool huge = !long_rows && uniform && stage_tiles >= (1LL << 19);
    const long long WANT_ITEMS = (long_rows || huge) ? 1024 : 2048;
    const int MAX_AUTO_SPAN = long_rows ? 4 : 8;
    if (!long_rows && st.cols > dbf_mfma_one_pass_cols()) return 4;
    long long item_tiles = stage_tiles / WANT_ITEMS;
    if (item_tiles > (huge ? 512 : 256)) item_tiles = huge ? 512 : 256;
    // (small stages: items of up to 48 KiB as long as that leaves a thousand of them -- 256 layers of 1024 x 4096 at
    //  1 / 1.5 / 2.3 bits per weight 4.05 / 4.52 / 5.19 -> 4.36 / 4.66 / 5.43 TB/s, 64 layers of 4096 x 4096, k = 2048
    //  4.35 -> 4.47)
    if (!long_rows) {
        const long long roomy = stage_tiles / 1024 < 48 ? stage_tiles / 1024 : 48;
        if (item_tiles < roomy) item_tiles = roomy;
    }
    int span = (int)((2 * item_tiles + st.n_ct) / (2 * st.n_ct));  // item_tiles / n_ct, rounded to nearest
    if (span < 1) span = 1;
    if (span > MAX_AUTO_SPAN) span = MAX_AUTO_SPAN;
    return span;
}

// The row tiles of a stage in as many items as `span` row tiles per item need, of equal length to within one row
// tile (32 row tiles at 5 per item: 5 5 5 5 4 4 4 instead of 5 5 5 5 5 5 2).
std::vector<int> balanced_spans(int n_rt, int span) {
    const int items = (n_rt + span - 1) / span, base = n_rt / items, longer = n_rt % items;
    std::vector<int> out;
    for (int q = 0; q < items; ++q) out.push_back(base + (q < longer ? 1 : 0));
    return out;
}

// The same for the launches of batches of 2 and more, which take a stage input quantised once per call: a workgroup
// starts on a copy of up to 52 KiB of int8 planes, two launches per stage leave more of a tail, and fewer, longer
// items did better: about 512 per stage, of equal length within a layer.  Measured on 512 layers of 4096 x 4096,
// k = 2048 at batch 2 / 4 / 8: 5.36 / 4.76 / 3.85 TB/s with 16 row tiles per item against 5.10 / 4.53 / 3.72 with
// 2 and 4 (768 items per stage: 5.30 / 4.50 / 3.75).
int shared_span(const DbfStage& st, long long stage_tiles) {
    constexpr long long WANT_ITEMS = 512;
    const long long item_tiles = stage_tiles / WANT_ITEMS;
    long long span = (2 * item_tiles + st.n_ct) / (2 * st.n_ct);
    if (span < 1) span = 1;
    if (span > DBF_MAX_SPAN) span = DBF_MAX_SPAN;
    const long long per_layer = (st.n_rt + span - 1) / span;  // items of equal length ...
    span = (st.n_rt + per_layer - 1) / per_layer;
    // ... in whole groups of four row tiles, one per wavefront, unless that leaves the stage with too few items to
    // fill the chip (8192 x 28672 streams of 19 layers at batch 4: 4.13 TB/s with 475 items of two row tiles, whose
    // wavefronts share the column tiles, against 3.74 with 247 items of four)
    if (span >= 2) {
        const long long up = (span + 3) & ~3ll, down = span & ~3ll;
        if (stage_tiles / (up * st.n_ct) >= 256) span = up;  // (at least one item per compute unit)
        else if (down >= 4) span = down;
    }
    return (int)(span > DBF_MAX_SPAN ? DBF_MAX_SPAN : span);
}

void free_plan(DbfPlan& p) {
    if (p.dev_block) (void)hipFree(p.dev_block);
    p.dev_block = nullptr;
}

// Builds and uploads the launch tables for `n` layers whose stages (with their x/y offsets
// already set) are given in sB / sA.
int build_plan(const std::vector<DbfStage>& sB, const std::vector<DbfStage>& sA, const std::vector<int>& span_b,
               const std::vector<int>& span_a, DbfPlan* p) {
    const int n = (int)sB.size();
    std::vector<DbfWorkItem> wB1, wA1;
    std::vector<DbfItem> items_n, items_1;
    int nBn = 0, nB1 = 0;
    std::memset(p, 0, sizeof(*p));
    for (int i = 0; i < n; ++i) {
        for (int rt = 0; rt < sB[i].n_rt; ++rt) wB1.push_back(DbfWorkItem{i, rt, 1, 0});
        for (int rt = 0; rt < sA[i].n_rt; ++rt) wA1.push_back(DbfWorkItem{i, rt, 1, 0});
        if (sB[i].cols > p->max_cols_B) p->max_cols_B = sB[i].cols;
        if (sA[i].cols > p->max_cols_A) p->max_cols_A = sA[i].cols;
    }
    // Several layers most of whose sign bytes sit in layers with long stage inputs -- one longer than the one-pass
    // prologue holds, so that every workgroup would read it twice (for the scale, then for the rounding: as many
    // bytes as a third to a half of the workgroup's signs), and the other longer than 4096: such plans quantise
    // every stage input once per call at every batch, in launches of their own.  Measured on streams of 0.5 GB:
    // 8192 x 28672 at 1 bit per weight 3.06 -> 4.7 TB/s, 8192 x 8192 at 2 bits 4.09 -> 5.0; with the other stage
    // short (8192 x 8192 or 4096 x 14336 at 1 bit) the one-launch path is as fast or faster (5.36 against 5.2 TB/s).
    {
        const int lr = dbf_tune(DBF_TUNE_LONG_ROWS);
        double bytes_long = 0, bytes_all = 0;
        for (int i = 0; i < n; ++i) {
            const int hi = sB[i].cols > sA[i].cols ? sB[i].cols : sA[i].cols;
            const int lo = sB[i].cols > sA[i].cols ? sA[i].cols : sB[i].cols;
            const double bytes = ((double)sB[i].n_rt * sB[i].n_ct + (double)sA[i].n_rt * sA[i].n_ct) * DBF_TILE_BYTES;
            bytes_all += bytes;
            if (hi > dbf_mfma_one_pass_cols() && lo > 4096) bytes_long += bytes;
        }
        p->long_rows = lr == 1 || (lr < 0 && n > 1 && 2 * bytes_long > bytes_all);
    }
    p->x_vec_ok = 1;
    for (int i = 0; i < n; ++i)
        if ((sB[i].cols & 7) != 0 || (sB[i].x_off & 7) != 0) p->x_vec_ok = 0;
    const std::vector<int> one(1, 1);
    // row tiles per item: the given pattern, or (empty pattern) chosen per layer from the size of the launch
    long long tiles_B = 0, tiles_A = 0;
    for (int i = 0; i < n; ++i) {
        tiles_B += (long long)sB[i].n_rt * sB[i].n_ct;
        tiles_A += (long long)sA[i].n_rt * sA[i].n_ct;
    }
    int max_span = 1;
    int phase = 0;
    bool uniform = true;  // every layer has the shape of the first
    for (int i = 1; i < n; ++i)
        if (sB[i].rows != sB[0].rows || sB[i].cols != sB[0].cols || sA[i].rows != sA[0].rows) uniform = false;
    auto pattern_for = [&](const std::vector<int>& given, const DbfStage& st, long long stage_tiles) {
        std::vector<int> v = given;
        if (given.empty()) {  // (a pattern of this layer's own: it starts at its first item)
            v = balanced_spans(st.n_rt, auto_span(st, stage_tiles, p->long_rows != 0, uniform));
            phase = 0;
        }
        for (int x : v) max_span = x > max_span ? x : max_span;
        return v;
    };
    for (int i = 0; i < n; ++i) append_items(items_n, sB[i], i, false, 0, pattern_for(span_b, sB[i], tiles_B), &phase);
    nBn = (int)items_n.size();
    phase = 0;
    for (int i = 0; i < n; ++i)
        append_items(items_n, sA[i], i, true, sB[i].n_rt, pattern_for(span_a, sA[i], tiles_A), &phase);
    // (the list of the launches that take a shared quantised input)
    auto shared_pattern_for = [&](const std::vector<int>& given, const DbfStage& st, long long stage_tiles) {
        std::vector<int> v = given.empty() ? std::vector<int>(1, shared_span(st, stage_tiles)) : given;
        for (int x : v) max_span = x > max_span ? x : max_span;
        return v;
    };
    std::vector<DbfItem> items_s;
    phase = 0;
    for (int i = 0; i < n; ++i) append_items(items_s, sB[i], i, false, 0, shared_pattern_for(span_b, sB[i], tiles_B), &phase);
    const int nBs = (int)items_s.size();
    phase = 0;
    for (int i = 0; i < n; ++i)
        append_items(items_s, sA[i], i, true, sB[i].n_rt, shared_pattern_for(span_a, sA[i], tiles_A), &phase);
    // Workgroups are handed to the 8 compute dies in turn (linear workgroup id modulo 8) and each die has an L2 of
    // its own.  In the lists of stacks the items of a layer are placed so that they run on ONE die, one after the
    // other: the layer's inputs (x and b, the middle activations) then come from that die's L2 for every item but
    // the first.  Layers are dealt to the dies by sign bytes; list position p of a launch belongs to die p mod 8, and
    // a die whose queue has run dry takes from the longest.  Only the order of the items changes (B items still
    // before A items, and a layer's items still in order).  Measured on one box: the 224-layer Llama-2-7B stack
    // 5.97 -> 6.03 TB/s, the 512-layer stream at batch 4 / 16 5.08 -> 5.10 / 3.32 -> 3.37, at batch 1 6.02 -> 6.01.
    if (n >= 16) {
        std::vector<int> die_of(n);
        double load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
        for (int i = 0; i < n; ++i) {
            int best = 0;
            for (int d = 1; d < 8; ++d)
                if (load[d] < load[best]) best = d;
            die_of[i] = best;
            load[best] += (double)sB[i].n_rt * sB[i].n_ct + (double)sA[i].n_rt * sA[i].n_ct;
        }
        // (`first`: the list position that is workgroup 0 of the launch the part runs in)
        auto by_die = [&](std::vector<DbfItem>& list, int begin, int end, int first) {
            std::vector<std::vector<DbfItem>> q(8);
            for (int pos = begin; pos < end; ++pos) q[die_of[list[pos].layer]].push_back(list[pos]);
            size_t at[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            for (int pos = begin; pos < end; ++pos) {
                int d = (pos - first) & 7;
                if (at[d] >= q[d].size()) {
                    size_t most = 0;
                    for (int e = 0; e < 8; ++e)
                        if (q[e].size() - at[e] > most) {
                            most = q[e].size() - at[e];
                            d = e;
                        }
                }
                list[pos] = q[d][at[d]++];
            }
        };
        // items_n runs as one launch (B and A items together) unless the plan quantises its inputs in launches of
        // their own; items_s always runs as a launch per stage
        by_die(items_n, 0, nBn, 0);
        by_die(items_n, nBn, (int)items_n.size(), p->long_rows ? nBn : 0);
        by_die(items_s, 0, nBs, 0);
        by_die(items_s, nBs, (int)items_s.size(), nBs);
    }
    phase = 0;
    for (int i = 0; i < n; ++i) append_items(items_1, sB[i], i, false, 0, one, &phase);
    nB1 = (int)items_1.size();
    for (int i = 0; i < n; ++i) append_items(items_1, sA[i], i, true, sB[i].n_rt, one, &phase);

    // Column pieces for launches with few row tiles.  Accumulators: int32 [DBF_PIECES_MAX_BATCH][rows of
    // the stage, padded to whole tiles] per layer and stage; counters: one per row tile.  Both start at
    // zero and are returned to zero by the workgroup that finishes a row tile.
    long long rtB = 0, rtA = 0;
    for (int i = 0; i < n; ++i) {
        rtB += sB[i].n_rt;
        rtA += sA[i].n_rt;
    }
    std::vector<int> pcB(n, 1), pcA(n, 1);
    bool cut = false;
    const int max_rt = dbf_tune(DBF_TUNE_PIECE_MAX_ROW_TILES);
    if (p->long_rows) {
        // (no pieces: the rows are cheap to start on, and whole row tiles per workgroup did better)
    } else if (rtB <= max_rt && rtA <= max_rt) {
        for (int i = 0; i < n; ++i) {
            pcB[i] = pieces_for(sB[i].n_ct, (int)rtB);
            pcA[i] = pieces_for(sA[i].n_ct, (int)rtA);
            cut = cut || pcB[i] > 1 || pcA[i] > 1;
        }
    }
    p->piece_row_tiles = (int)(rtB > rtA ? rtB : rtA);
    const size_t acc_ints = cut ? (size_t)DBF_PIECES_MAX_BATCH * DBF_TILE_ROWS * (size_t)(rtB + rtA) : 0;
    const size_t cnt_ints = cut ? (size_t)(rtB + rtA) * DBF_PIECE_CNT_STRIDE : 0;

    size_t off = 0;
    const size_t o_sB = off;  off = align_up(off + sizeof(DbfStage) * n, 256);
    const size_t o_sA = off;  off = align_up(off + sizeof(DbfStage) * n, 256);
    const size_t o_wB = off;  off = align_up(off + sizeof(DbfWorkItem) * wB1.size(), 256);
    const size_t o_wA = off;  off = align_up(off + sizeof(DbfWorkItem) * wA1.size(), 256);
    const size_t o_in = off;  off = align_up(off + sizeof(DbfItem) * items_n.size(), 256);
    const size_t o_i1 = off;  off = align_up(off + sizeof(DbfItem) * items_1.size(), 256);
    const size_t o_is = off;  off = align_up(off + sizeof(DbfItem) * items_s.size(), 256);
    const size_t o_sy = off;  off = align_up(off + sizeof(unsigned long long) * (2 * (size_t)n + 1) * DBF_SYNC_STRIDE, 256);
    const size_t o_ac = off;  off = align_up(off + sizeof(int) * acc_ints, 256);
    const size_t o_cn = off;  off = align_up(off + sizeof(int) * cnt_ints, 256);
    std::vector<DbfItem> items_p;
    int nBp = 0;
    if (cut) {
        // device addresses are offsets from the block's base, known only after the allocation:
        // build with a null base here and rebase below
        int* acc0 = reinterpret_cast<int*>(o_ac);
        int* cnt0 = reinterpret_cast<int*>(o_cn);
        size_t row_tiles_before = 0;
        for (int i = 0; i < n; ++i) {
            const int stride = sB[i].n_rt * DBF_TILE_ROWS;
            append_piece_items(items_p, sB[i], i, false, 0, pcB[i],
                               acc0 + (size_t)DBF_PIECES_MAX_BATCH * DBF_TILE_ROWS * row_tiles_before, stride,
                               cnt0 + (size_t)row_tiles_before * DBF_PIECE_CNT_STRIDE);
            row_tiles_before += sB[i].n_rt;
        }
        nBp = (int)items_p.size();
        for (int i = 0; i < n; ++i) {
            const int stride = sA[i].n_rt * DBF_TILE_ROWS;
            append_piece_items(items_p, sA[i], i, true, sB[i].n_rt, pcA[i],
                               acc0 + (size_t)DBF_PIECES_MAX_BATCH * DBF_TILE_ROWS * row_tiles_before, stride,
                               cnt0 + (size_t)row_tiles_before * DBF_PIECE_CNT_STRIDE);
            row_tiles_before += sA[i].n_rt;
        }
    }
    // what one launch adds to a layer's counters, in every item of every list
    for (std::vector<DbfItem>* list : {&items_n, &items_1, &items_s, &items_p})
        for (DbfItem& it : *list) {
            it.need = sB[it.layer].n_rt;
            it.peers = sA[it.layer].n_rt;
        }
    const size_t o_ip = off;  off = align_up(off + sizeof(DbfItem) * items_p.size(), 256);
    std::vector<uint8_t> image(off, 0);
    std::memcpy(image.data() + o_sB, sB.data(), sizeof(DbfStage) * n);
    std::memcpy(image.data() + o_sA, sA.data(), sizeof(DbfStage) * n);
    std::memcpy(image.data() + o_wB, wB1.data(), sizeof(DbfWorkItem) * wB1.size());
    std::memcpy(image.data() + o_wA, wA1.data(), sizeof(DbfWorkItem) * wA1.size());
    std::memcpy(image.data() + o_in, items_n.data(), sizeof(DbfItem) * items_n.size());
    std::memcpy(image.data() + o_i1, items_1.data(), sizeof(DbfItem) * items_1.size());
    std::memcpy(image.data() + o_is, items_s.data(), sizeof(DbfItem) * items_s.size());
    void* dev = nullptr;
    hipError_t e = dbf_mfma_prepare();
    if (e == hipSuccess) e = hipMalloc(&dev, off);
    if (e == hipSuccess) {
        for (DbfItem& it : items_p) {  // rebase the accumulator and counter addresses
            it.acc = reinterpret_cast<int*>(static_cast<uint8_t*>(dev) + reinterpret_cast<size_t>(it.acc));
            it.cnt = reinterpret_cast<int*>(static_cast<uint8_t*>(dev) + reinterpret_cast<size_t>(it.cnt));
        }
        std::memcpy(image.data() + o_ip, items_p.data(), sizeof(DbfItem) * items_p.size());
    }
    if (e == hipSuccess) e = hipMemcpy(dev, image.data(), off, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        (void)hipGetLastError();
        if (dev) (void)hipFree(dev);
        return DBF_EHIP;
    }
    uint8_t* d = static_cast<uint8_t*>(dev);
    p->dev_block = dev;
    p->n_layers = n;
    p->d_stagesB = reinterpret_cast<DbfStage*>(d + o_sB);
    p->d_stagesA = reinterpret_cast<DbfStage*>(d + o_sA);
    p->d_workB1 = reinterpret_cast<DbfWorkItem*>(d + o_wB);
    p->d_workA1 = reinterpret_cast<DbfWorkItem*>(d + o_wA);
    p->blocksB1 = (int)wB1.size();
    p->blocksA1 = (int)wA1.size();
    p->d_items_n = reinterpret_cast<DbfItem*>(d + o_in);
    p->nBn = nBn;
    p->nAn = (int)items_n.size() - nBn;
    p->d_items_1 = reinterpret_cast<DbfItem*>(d + o_i1);
    p->nB1 = nB1;
    p->nA1 = (int)items_1.size() - nB1;
    p->d_items_s = reinterpret_cast<DbfItem*>(d + o_is);
    p->nBs = nBs;
    p->nAs = (int)items_s.size() - nBs;
    p->rows_ok = 2 * (rtB + rtA) >= 7 * (long long)items_s.size();  // at least 3.5 row tiles per item on average
    p->d_sync = reinterpret_cast<unsigned long long*>(d + o_sy);
    p->d_items_p = cut ? reinterpret_cast<DbfItem*>(d + o_ip) : nullptr;
    p->nBp = nBp;
    p->nAp = (int)items_p.size() - nBp;
    p->span = max_span;
    return DBF_OK;
}

// Section offsets of a layer's single device block (256-byte aligned sections).
struct LayerOffsets {
    size_t A, B, a, m, b, image_bytes, t, qB, qA, total;
    int a_len, m_len, b_len, t_stride;
};
LayerOffsets layer_offsets(int n_in, int n_out, int k) {
    LayerOffsets o;
    o.a_len = dbf_row_tiles(n_out) * DBF_TILE_ROWS;
    o.m_len = dbf_row_tiles(k) * DBF_TILE_ROWS;
    o.b_len = dbf_col_tiles(n_in) * DBF_TILE_COLS;
    o.t_stride = o.m_len;  // >= col_tiles(k)*64, so the A stage may read its padded columns
    size_t off = 0;
    o.A = off;  off = align_up(off + dbf_tiled_bytes(n_out, k), 256);
    o.B = off;  off = align_up(off + dbf_tiled_bytes(k, n_in), 256);
    o.a = off;  off = align_up(off + 2 * (size_t)o.a_len, 256);
    o.m = off;  off = align_up(off + 2 * (size_t)o.m_len, 256);
    o.b = off;  off = align_up(off + 2 * (size_t)o.b_len, 256);
    o.image_bytes = off;  // signs and vectors; the scratch follows
    o.t = off;  off = align_up(off + 4 * (size_t)DBF_MAX_BATCH * o.t_stride, 256);
    o.qB = off;  off = align_up(off + DBF_QIN_HEADER + 2 * (size_t)DBF_MAX_BATCH * o.b_len, 256);
    o.qA = off;  off = align_up(off + DBF_QIN_HEADER + 2 * (size_t)DBF_MAX_BATCH * dbf_col_tiles(k) * DBF_TILE_COLS, 256);
    o.total = off;
    return o;
}

// Allocates the device block of a layer of the given shape on the current device and describes it
// (pointers, stages); the contents are left to the caller except the scratch, which is zeroed.
int create_layer(int n_in, int n_out, int k, const LayerOffsets& o, dbf_layer** out) {
    dbf_layer* L = new (std::nothrow) dbf_layer();
    if (!L) return DBF_ENOMEM;
    void* dev = nullptr;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess || hipMalloc(&dev, o.total) != hipSuccess) {
        (void)hipGetLastError();
        delete L;
        return DBF_EHIP;
    }
    if (hipMemset(static_cast<uint8_t*>(dev) + o.t, 0, o.total - o.t) != hipSuccess) {
        (void)hipGetLastError();
        (void)hipFree(dev);
        delete L;
        return DBF_EHIP;
    }
    uint8_t* d = static_cast<uint8_t*>(dev);
    L->n_in = n_in;  L->n_out = n_out;  L->k = k;  L->device = device;
    L->dev_block = dev;  L->device_bytes = o.total;
    L->dA = d + o.A;  L->dB = d + o.B;
    L->da = reinterpret_cast<uint16_t*>(d + o.a);
    L->dm = reinterpret_cast<uint16_t*>(d + o.m);
    L->db = reinterpret_cast<uint16_t*>(d + o.b);
    L->dt = reinterpret_cast<float*>(d + o.t);
    L->t_stride = o.t_stride;
    L->dqB = d + o.qB;
    L->dqA = d + o.qA;

    DbfStage& sb = L->h_stages[0];
    sb.bits = L->dB;  sb.in_scale = L->db;  sb.row_scale = L->dm;  sb.t = L->dt;
    sb.x_off = 0;  sb.y_off = 0;
    sb.n_rt = dbf_row_tiles(k);  sb.n_ct = dbf_col_tiles(n_in);
    sb.rows = k;  sb.cols = n_in;  sb.t_stride = o.t_stride;  sb.pad_ = 0;  sb.q_in = L->dqB;
    DbfStage& sa = L->h_stages[1];
    sa.bits = L->dA;  sa.in_scale = nullptr;  sa.row_scale = L->da;  sa.t = L->dt;
    sa.x_off = 0;  sa.y_off = 0;
    sa.n_rt = dbf_row_tiles(n_out);  sa.n_ct = dbf_col_tiles(k);
    sa.rows = n_out;  sa.cols = k;  sa.t_stride = o.t_stride;  sa.pad_ = 0;  sa.q_in = L->dqA;
    *out = L;
    return DBF_OK;
}

// The launch plan of a layer alone: one row tile per workgroup gives the most parallelism.
int finish_layer(dbf_layer* L) {
    std::vector<DbfStage> vB(1, L->h_stages[0]), vA(1, L->h_stages[1]);
    return build_plan(vB, vA, std::vector<int>(1, 1), std::vector<int>(1, 1), &L->plan);
}

void destroy_layer(dbf_layer* L) {
    if (!L) return;
    free_plan(L->plan);
    if (L->dev_block) (void)hipFree(L->dev_block);
    delete L;
}

// Builds the device image of a layer from canonical words and uploads it.
int build_layer(int n_in, int n_out, int k, const uint32_t* A_bits, const uint32_t* B_bits,
                const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out) {
    const LayerOffsets o = layer_offsets(n_in, n_out, k);
    uint8_t* image = static_cast<uint8_t*>(std::calloc(o.image_bytes, 1));
    if (!image) return DBF_ENOMEM;
    int rc = dbf_tile_host(n_out, k, A_bits, image + o.A);
    if (rc == DBF_OK) rc = dbf_tile_host(k, n_in, B_bits, image + o.B);
    if (rc != DBF_OK) {
        std::free(image);
        return rc;
    }
    std::memcpy(image + o.a, a, 2 * (size_t)n_out);
    std::memcpy(image + o.m, m, 2 * (size_t)k);
    std::memcpy(image + o.b, b, 2 * (size_t)n_in);

    dbf_layer* L = nullptr;
    rc = create_layer(n_in, n_out, k, o, &L);
    if (rc != DBF_OK) {
        std::free(image);
        return rc;
    }
    hipError_t e = hipMemcpy(L->dev_block, image, o.image_bytes, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    std::free(image);
    if (e != hipSuccess || finish_layer(L) != DBF_OK) {
        (void)hipGetLastError();
        destroy_layer(L);
        return DBF_EHIP;
    }
    *out = L;
    return DBF_OK;
}

inline bool kind_ok(int kind) {
    return kind == DBF_GEMV_AUTO || kind == DBF_GEMV_VALU || kind == DBF_GEMV_MFMA || kind == DBF_GEMV_MFMA_SPLIT;
}

// Launches one decode pass of a plan on `stream`.  `mid`, if not NULL, is recorded between the
// B-stage launch and the A-stage launch of the two-launch kinds (timed entry point only).
int launch_plan(int kind, const DbfPlan& p, const void* x, void* y, int batch, hipStream_t stream,
                hipEvent_t mid = nullptr) {
    // AUTO: one fused launch for both stages only where the B items alone fill the chip (DBF_TUNE_FUSED_MIN_B_ITEMS), else
    // a launch per stage.  In a short list every A item is resident from the start and sits polling its layer's
    // counter next to the B items it waits for.  Per call, one launch against two, us:
    //   4096 x 4096, k = 2048    1 layer 12.0 / 11.0   3: 12.3 / 11.2   8: 12.6 / 11.3   24: 20.5 / 16.6   48: 27.3 / 22.8
    //                            56 (896 B items): 28.6 / 26.7   64 (1024): 27.0 / 27.6   96: 39.6 / 40.8   128: 52.0 / 53.5
    //   4096 -> 11008, k = 2985  3 layers 15.4 / 13.6   24: 34.3 / 32.8   40 (960 B items): 43.5 / 44.5   56: 59.7 / 62.2
    //                            128: 122.8 / 128.6
    // (with the layers' counters side by side in memory instead of 512 bytes apart the one launch took 19.4 us at 8
    //  layers, 42.9 at 24, 88 at 24 layers of the second shape: every poll went to the same memory channel)
    // Stage inputs too long for exact int32 sums (DBF_INT_PATH_MAX_COLS): the vector-ALU kernel, or an error for the
    // kinds that name the matrix-core kernel.
    const int longest = p.max_cols_B > p.max_cols_A ? p.max_cols_B : p.max_cols_A;
    if (longest > DBF_INT_PATH_MAX_COLS) {
        if (kind == DBF_GEMV_MFMA || kind == DBF_GEMV_MFMA_SPLIT) return DBF_ESHAPE;
        kind = DBF_GEMV_VALU;
    }
    const int FUSED_MIN_B_ITEMS = dbf_tune(DBF_TUNE_FUSED_MIN_B_ITEMS);
    const bool pieces_ok = kind == DBF_GEMV_AUTO;  // the named kinds keep their one-workgroup-per-row-tile lists
    if (kind == DBF_GEMV_AUTO) kind = DBF_GEMV_MFMA_SPLIT;  // (until the list is known, below)
    const int wait_us = dbf_tune(DBF_TUNE_WAIT_LIMIT_US);
    if (kind == DBF_GEMV_VALU) {
        DBF_HIP_TRY(dbf_launch_stage_valu(false, p.d_stagesB, p.d_workB1, p.blocksB1, x, y, batch, stream));
        if (mid) DBF_HIP_TRY(hipEventRecord(mid, stream));
        DBF_HIP_TRY(dbf_launch_stage_valu(true, p.d_stagesA, p.d_workA1, p.blocksA1, x, y, batch, stream));
        return DBF_OK;
    }
    // several row tiles per workgroup only if all columns of both stages fit one LDS chunk
    const int max_cols = p.max_cols_B > p.max_cols_A ? p.max_cols_B : p.max_cols_A;
    // (column pieces at batch 2 only for a layer or three.  Wide rows, us per call with / without pieces at
    //  batch 2: 1 layer of 11008 -> 4096 23.5 / 26.8, 3 layers 26.9 / 27.0, 4 layers 27.8 / 24.6, 8: 31.3 / 26.0,
    //  16: 51.0 / 30.9, 32: 113.8 / 48.8)
    const bool use_pieces = pieces_ok && p.d_items_p && !p.long_rows &&
                            (batch == 1 || (batch <= DBF_PIECES_MAX_BATCH && p.piece_row_tiles <= 96));
    // Batches of 2 and more: every stage input is quantised once per call; the items read it from memory tile by tile,
    // in the ring of the sign tiles (2), with a row tile per wavefront where the list has long items (3).
    int shared_q = 0;
    if (pieces_ok && !use_pieces && (batch >= dbf_tune(DBF_TUNE_SHARED_MIN_BATCH) || p.long_rows)) {
        // (the LDS copy, form 1, is left to the knob: where the operand fits LDS -- batch 2-4 at 4096 columns -- reading
        //  it from memory with the tiles was faster on every list that is too short for form 3: a layer alone at batch
        //  2 / 3 / 4 17.1 / 18.4 / 19.3 -> 15.0 / 15.6 / 15.7 us, 16 layers 18.7 / 19.7 / 20.4 -> 17.9 / 18.2 / 18.5,
        //  32 layers of 4096 -> 11008 51.4 / 53.3 / 54.0 -> 48.1 / 50.4 / 51.5)
        //  (long-rows plans at batch 1 too: 4096 x 14336 and 8192 x 8192 streams ran 2-5 % faster than with the copy)
        shared_q = 2;
        // (a list of long items: a row tile per wavefront, the four wavefronts of a workgroup reading the same
        //  operand from memory at the same time.  512 layers of 4096 x 4096, k = 2048: 5.63 / 5.27 / 4.61 / 3.34 TB/s
        //  at batch 2 / 4 / 8 / 16 against 5.42 / 4.80 with the LDS copy and 3.98 / 2.60 with every wavefront
        //  reading the operand of its own column tiles)
        if (batch >= 2 && p.rows_ok) shared_q = 3;
        if (dbf_tune(DBF_TUNE_SHARED_Q) >= 0) shared_q = dbf_tune(DBF_TUNE_SHARED_Q);
    }
    const bool span = dbf_mfma_chunk_tiles(batch, max_cols, shared_q) >= dbf_col_tiles(max_cols);
    const bool long_list = shared_q && batch >= 2;  // fewer, longer items (shared_span)
    const DbfItem* items = !span ? p.d_items_1 : long_list ? p.d_items_s : p.d_items_n;
    int nB = !span ? p.nB1 : long_list ? p.nBs : p.nBn, nA = !span ? p.nA1 : long_list ? p.nAs : p.nAn;
    int pieces = 0;
    if (use_pieces) {  // few row tiles: cut them into column pieces
        items = p.d_items_p;
        nB = p.nBp;
        nA = p.nAp;
        pieces = 1;
    }
    if (pieces_ok && p.n_layers > 1 && nB >= FUSED_MIN_B_ITEMS) kind = DBF_GEMV_MFMA;
    // (batch 1: can every x row be read in 16-byte pieces?  Then rows of up to 6144 columns all take the one-pass prologue)
    const int one_pass_rows = batch == 1 && p.x_vec_ok && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
    if (shared_q) {
        // Four launches: quantise x, B items, quantise t, A items.
        DBF_HIP_TRY(dbf_launch_quantise_inputs(p.d_stagesB, p.n_layers, 0, x, batch, stream));
        DBF_HIP_TRY(dbf_launch_items_mfma(items, nB, p.d_sync, p.n_layers, 0, x, y, batch, max_cols, 0, shared_q, 0, wait_us, stream));
        if (mid) DBF_HIP_TRY(hipEventRecord(mid, stream));
        DBF_HIP_TRY(dbf_launch_quantise_inputs(p.d_stagesA, p.n_layers, 1, x, batch, stream));
        DBF_HIP_TRY(dbf_launch_items_mfma(items + nB, nA, p.d_sync, p.n_layers, 0, x, y, batch, max_cols, 0, shared_q, 0, wait_us, stream));
        return DBF_OK;
    }
    if (kind == DBF_GEMV_MFMA) {
        DBF_HIP_TRY(dbf_launch_items_mfma(items, nB + nA, p.d_sync, p.n_layers, 1, x, y, batch, max_cols, pieces, 0, one_pass_rows, wait_us, stream));
        if (mid) DBF_HIP_TRY(hipEventRecord(mid, stream));
        return DBF_OK;
    }
    DBF_HIP_TRY(dbf_launch_items_mfma(items, nB, p.d_sync, p.n_layers, 0, x, y, batch, max_cols, pieces, 0, one_pass_rows, wait_us, stream));
    if (mid) DBF_HIP_TRY(hipEventRecord(mid, stream));
    DBF_HIP_TRY(dbf_launch_items_mfma(items + nB, nA, p.d_sync, p.n_layers, 0, x, y, batch, max_cols, pieces, 0, one_pass_rows, wait_us, stream));
    return DBF_OK;
}

int read_timeouts(const DbfPlan& p, int* timeouts) {
    unsigned long long v = 0;
    DBF_HIP_TRY(hipDeviceSynchronize());
    DBF_HIP_TRY(hipMemcpy(&v, p.d_sync + (size_t)(2 * p.n_layers) * DBF_SYNC_STRIDE, sizeof(v), hipMemcpyDeviceToHost));
    if (timeouts) *timeouts = v > 0x7fffffffull ? 0x7fffffff : (int)v;
    return DBF_OK;
}

// Row tiles per workgroup in stack launches: the tuning knob's fixed value, or (0) empty, which lets
// build_plan choose per layer from the size of the launch (auto_span).  The input vector is quantised once
// per workgroup, so larger items amortise that prologue and smaller ones balance the end of the launch.
std::vector<int> stack_spans(int knob) {
    const int v = dbf_tune(knob);
    return v > 0 ? std::vector<int>(1, v) : std::vector<int>();
}

}  // namespace

extern "C" {

size_t dbf_gemm_workspace_bytes(const dbf_layer* L, int T) {
    if (!L || T < 1) return 0;
    return dbf_gemm_i8_workspace_bytes(L, T);
}

int dbf_gemm_kind(const dbf_layer* L, const void* X_dev, void* Y_dev, int T, void* workspace_dev,
                  size_t workspace_bytes, int kind, void* hip_stream) {
    if (!L || !X_dev || !Y_dev || T < 1) return DBF_EINVAL;
    if (kind != DBF_GEMM_AUTO && kind != DBF_GEMM_I8) return DBF_EINVAL;
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) ||
        workspace_bytes < dbf_gemm_workspace_bytes(L, T))
        return DBF_EWORKSPACE;
    if ((T + 63) / 64 > 65535) return DBF_EINVAL;  // token blocks are the grid's y dimension
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // Up to 16 tokens are a decode batch: the same fixed-point arithmetic (the int8 prefill gives the decode
    // kernel's bits), at a third of the latency (a prefill workgroup walks all column steps of its rows
    // whatever the token count: 67 us against 24 us at 4096 x 4096, k = 4096).
    // Up to 32 tokens are two such batches, one after the other (4096 x 4096, k = 4096: 35-46 us for 17-32 tokens
    // against 64-65; 11008 -> 4096, k = 5970: 53-67 against 119-120; at 48 tokens three batches lose on the first).
    if (kind == DBF_GEMM_AUTO && T <= 2 * DBF_MAX_BATCH) {
        for (int t0 = 0; t0 < T; t0 += DBF_MAX_BATCH) {
            const int nb = T - t0 < DBF_MAX_BATCH ? T - t0 : DBF_MAX_BATCH;
            const int rc = launch_plan(DBF_GEMV_AUTO, L->plan, static_cast<const uint16_t*>(X_dev) + (size_t)t0 * L->n_in,
                                       static_cast<uint16_t*>(Y_dev) + (size_t)t0 * L->n_out, nb, stream);
            if (rc != DBF_OK) return rc;
        }
        return DBF_OK;
    }
    if (L->n_in > DBF_INT_PATH_MAX_COLS || L->k > DBF_INT_PATH_MAX_COLS) return DBF_ESHAPE;  // (int32 sums: see dbf.h)
    const hipError_t e = dbf_gemm_i8_launch(L, X_dev, Y_dev, T, workspace_dev, workspace_bytes, stream);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return DBF_EHIP;
    }
    return DBF_OK;
}

int dbf_gemm(const dbf_layer* L, const void* X_dev, void* Y_dev, int T, void* workspace_dev,
             size_t workspace_bytes, void* hip_stream) {
    return dbf_gemm_kind(L, X_dev, Y_dev, T, workspace_dev, workspace_bytes, DBF_GEMM_AUTO, hip_stream);
}

int dbf_pack_bits(int n_in, int n_out, int k, const uint32_t* A_bits, const uint32_t* B_bits,
                  const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out) {
    if (out) *out = nullptr;
    if (!A_bits || !B_bits || !a || !m || !b || !out) return DBF_EINVAL;
    if (!shape_ok(n_in, n_out, k)) return DBF_ESHAPE;
    return build_layer(n_in, n_out, k, A_bits, B_bits, a, m, b, out);
}

int dbf_pack(int n_in, int n_out, int k, const int8_t* A_pm1, const int8_t* B_pm1,
             const uint16_t* a, const uint16_t* m, const uint16_t* b, dbf_layer** out) {
    if (out) *out = nullptr;
    if (!A_pm1 || !B_pm1 || !a || !m || !b || !out) return DBF_EINVAL;
    if (!shape_ok(n_in, n_out, k)) return DBF_ESHAPE;
    const size_t wa = (size_t)n_out * ((k + 31) / 32), wb = (size_t)k * ((n_in + 31) / 32);
    uint32_t* Ab = static_cast<uint32_t*>(std::malloc(wa * 4));
    uint32_t* Bb = static_cast<uint32_t*>(std::malloc(wb * 4));
    int rc = (Ab && Bb) ? DBF_OK : DBF_ENOMEM;
    if (rc == DBF_OK) rc = dbf_signs_to_bits_host(n_out, k, A_pm1, Ab);
    if (rc == DBF_OK) rc = dbf_signs_to_bits_host(k, n_in, B_pm1, Bb);
    if (rc == DBF_OK) rc = build_layer(n_in, n_out, k, Ab, Bb, a, m, b, out);
    std::free(Ab);
    std::free(Bb);
    return rc;
}

int dbf_unpack_bits(const dbf_layer* L, uint32_t* A_bits, uint32_t* B_bits, uint16_t* a,
                    uint16_t* m, uint16_t* b) {
    if (!L) return DBF_EINVAL;
    DBF_HIP_TRY(hipDeviceSynchronize());
    if (A_bits) {
        std::vector<uint8_t> img(dbf_tiled_bytes(L->n_out, L->k));
        DBF_HIP_TRY(hipMemcpy(img.data(), L->dA, img.size(), hipMemcpyDeviceToHost));
        const int rc = dbf_untile_host(L->n_out, L->k, img.data(), A_bits);
        if (rc != DBF_OK) return rc;
    }
    if (B_bits) {
        std::vector<uint8_t> img(dbf_tiled_bytes(L->k, L->n_in));
        DBF_HIP_TRY(hipMemcpy(img.data(), L->dB, img.size(), hipMemcpyDeviceToHost));
        const int rc = dbf_untile_host(L->k, L->n_in, img.data(), B_bits);
        if (rc != DBF_OK) return rc;
    }
    if (a) DBF_HIP_TRY(hipMemcpy(a, L->da, 2 * (size_t)L->n_out, hipMemcpyDeviceToHost));
    if (m) DBF_HIP_TRY(hipMemcpy(m, L->dm, 2 * (size_t)L->k, hipMemcpyDeviceToHost));
    if (b) DBF_HIP_TRY(hipMemcpy(b, L->db, 2 * (size_t)L->n_in, hipMemcpyDeviceToHost));
    return DBF_OK;
}

int dbf_dims(const dbf_layer* L, int* n_in, int* n_out, int* k, size_t* device_bytes) {
    if (!L) return DBF_EINVAL;
    if (n_in) *n_in = L->n_in;
    if (n_out) *n_out = L->n_out;
    if (k) *k = L->k;
    if (device_bytes) *device_bytes = L->device_bytes;
    return DBF_OK;
}

void dbf_free(dbf_layer* L) { destroy_layer(L); }

int dbf_prune_middle(const dbf_layer* L, const int32_t* keep, int n_keep, dbf_layer** out) {
    if (out) *out = nullptr;
    if (!L || !keep || !out || n_keep < 1 || n_keep > L->k) return DBF_EINVAL;
    for (int i = 0; i < n_keep; ++i)
        if (keep[i] < 0 || keep[i] >= L->k || (i > 0 && keep[i] <= keep[i - 1])) return DBF_EINVAL;
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) {
        (void)hipGetLastError();
        return DBF_EHIP;
    }
    if (device != L->device) return DBF_EINVAL;  // the new layer lives where the old one does

    dbf_layer* N = nullptr;
    const LayerOffsets o = layer_offsets(L->n_in, L->n_out, n_keep);
    int rc = create_layer(L->n_in, L->n_out, n_keep, o, &N);
    if (rc != DBF_OK) return rc;
    int* keep_dev = nullptr;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(&keep_dev), sizeof(int) * (size_t)n_keep);
    if (e == hipSuccess) e = hipMemcpy(keep_dev, keep, sizeof(int) * (size_t)n_keep, hipMemcpyHostToDevice);
    if (e == hipSuccess) e = dbf_prune_launch(L, N, keep_dev, n_keep, nullptr);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (keep_dev) (void)hipFree(keep_dev);
    if (e != hipSuccess || finish_layer(N) != DBF_OK) {
        (void)hipGetLastError();
        destroy_layer(N);
        return DBF_EHIP;
    }
    *out = N;
    return DBF_OK;
}

int dbf_gemv_kind(const dbf_layer* L, const void* x_dev, void* y_dev, int batch, int kind,
                  void* hip_stream) {
    if (!L || !x_dev || !y_dev) return DBF_EINVAL;
    if (batch < 1 || batch > DBF_MAX_BATCH || !kind_ok(kind)) return DBF_EINVAL;
    return launch_plan(kind, L->plan, x_dev, y_dev, batch, static_cast<hipStream_t>(hip_stream));
}

int dbf_gemv(const dbf_layer* L, const void* x_dev, void* y_dev, int batch, void* hip_stream) {
    return dbf_gemv_kind(L, x_dev, y_dev, batch, DBF_GEMV_AUTO, hip_stream);
}

int dbf_sync_timeouts(const dbf_layer* L, int* timeouts) {
    if (!L) return DBF_EINVAL;
    return read_timeouts(L->plan, timeouts);
}

// ---- stacks ---------------------------------------------------------------------------------

int dbf_stack_create_grouped(const dbf_layer* const* layers, int n_layers, const int* group_sizes, int n_groups,
                             dbf_stack** out) {
    if (out) *out = nullptr;
    if (!layers || !out || n_layers < 1) return DBF_EINVAL;
    for (int i = 0; i < n_layers; ++i)
        if (!layers[i]) return DBF_EINVAL;
    for (int i = 1; i < n_layers; ++i)
        if (layers[i]->device != layers[0]->device) return DBF_EINVAL;
    {   // a layer may appear only once: its scratch would be shared by two products of one launch
        std::vector<const dbf_layer*> sorted(layers, layers + n_layers);
        std::sort(sorted.begin(), sorted.end());
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return DBF_EINVAL;
    }
    // group of every layer: consecutive layers that read one input block
    std::vector<int> first_of(n_layers);
    if (group_sizes) {
        if (n_groups < 1) return DBF_EINVAL;
        int at = 0;
        for (int g = 0; g < n_groups; ++g) {
            if (group_sizes[g] < 1 || group_sizes[g] > n_layers - at) return DBF_EINVAL;
            for (int j = 0; j < group_sizes[g]; ++j) {
                if (layers[at + j]->n_in != layers[at]->n_in) return DBF_ESHAPE;
                first_of[at + j] = at;
            }
            at += group_sizes[g];
        }
        if (at != n_layers) return DBF_EINVAL;
    } else {
        for (int i = 0; i < n_layers; ++i) first_of[i] = i;
    }

    dbf_stack* S = new (std::nothrow) dbf_stack();
    if (!S) return DBF_ENOMEM;
    std::vector<DbfStage> sB(n_layers), sA(n_layers);
    S->h_x_prefix = static_cast<long long*>(std::malloc(sizeof(long long) * (n_layers + 1)));
    S->h_y_prefix = static_cast<long long*>(std::malloc(sizeof(long long) * (n_layers + 1)));
    if (!S->h_x_prefix || !S->h_y_prefix) {
        dbf_stack_free(S);
        return DBF_ENOMEM;
    }
    S->n_layers = n_layers;
    S->device = layers[0]->device;
    S->h_x_prefix[0] = S->h_y_prefix[0] = 0;
    long long x_end = 0;  // elements of x (per unit of batch) used so far
    for (int i = 0; i < n_layers; ++i) {
        const dbf_layer* L = layers[i];
        if (first_of[i] == i) {
            S->h_x_prefix[i] = x_end;
            x_end += L->n_in;
        } else {
            S->h_x_prefix[i] = S->h_x_prefix[first_of[i]];
        }
        sB[i] = L->h_stages[0];
        sA[i] = L->h_stages[1];
        sB[i].x_off = sA[i].x_off = S->h_x_prefix[i];
        sB[i].y_off = sA[i].y_off = S->h_y_prefix[i];
        S->h_y_prefix[i + 1] = S->h_y_prefix[i] + L->n_out;
    }
    S->h_x_prefix[n_layers] = x_end;
    const int rc = build_plan(sB, sA, stack_spans(DBF_TUNE_STACK_SPAN_B), stack_spans(DBF_TUNE_STACK_SPAN_A), &S->plan);
    if (rc != DBF_OK) {
        dbf_stack_free(S);
        return rc;
    }
    *out = S;
    return DBF_OK;
}

int dbf_stack_create(const dbf_layer* const* layers, int n_layers, dbf_stack** out) {
    return dbf_stack_create_grouped(layers, n_layers, nullptr, 0, out);
}

int dbf_stack_offsets(const dbf_stack* S, int layer_index, int batch, size_t* x_off, size_t* y_off) {
    if (!S || layer_index < 0 || layer_index > S->n_layers) return DBF_EINVAL;
    if (batch < 1 || batch > DBF_MAX_BATCH) return DBF_EINVAL;
    if (x_off) *x_off = (size_t)S->h_x_prefix[layer_index] * batch;
    if (y_off) *y_off = (size_t)S->h_y_prefix[layer_index] * batch;
    return DBF_OK;
}

int dbf_stack_gemv(const dbf_stack* S, const void* x_dev, void* y_dev, int batch, int kind,
                   void* hip_stream) {
    if (!S || !x_dev || !y_dev) return DBF_EINVAL;
    if (batch < 1 || batch > DBF_MAX_BATCH || !kind_ok(kind)) return DBF_EINVAL;
    return launch_plan(kind, S->plan, x_dev, y_dev, batch, static_cast<hipStream_t>(hip_stream));
}

int dbf_stack_gemv_timed(const dbf_stack* S, const void* x_dev, void* y_dev, int batch, int kind,
                         void* hip_stream, float* ms_first, float* ms_second) {
    if (!S || !x_dev || !y_dev) return DBF_EINVAL;
    if (batch < 1 || batch > DBF_MAX_BATCH || !kind_ok(kind)) return DBF_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    int rc = DBF_OK;
    for (int i = 0; i < 3 && rc == DBF_OK; ++i)
        if (hipEventCreate(&ev[i]) != hipSuccess) rc = DBF_EHIP;
    if (rc == DBF_OK && hipEventRecord(ev[0], stream) != hipSuccess) rc = DBF_EHIP;
    if (rc == DBF_OK) rc = launch_plan(kind, S->plan, x_dev, y_dev, batch, stream, ev[1]);
    if (rc == DBF_OK && hipEventRecord(ev[2], stream) != hipSuccess) rc = DBF_EHIP;
    if (rc == DBF_OK && hipEventSynchronize(ev[2]) != hipSuccess) rc = DBF_EHIP;
    float mb = 0.f, ma = 0.f;
    if (rc == DBF_OK && hipEventElapsedTime(&mb, ev[0], ev[1]) != hipSuccess) rc = DBF_EHIP;
    if (rc == DBF_OK && hipEventElapsedTime(&ma, ev[1], ev[2]) != hipSuccess) rc = DBF_EHIP;
    for (int i = 0; i < 3; ++i)
        if (ev[i]) (void)hipEventDestroy(ev[i]);
    if (rc != DBF_OK) (void)hipGetLastError();
    if (ms_first) *ms_first = mb;
    if (ms_second) *ms_second = ma;
    return rc;
}

int dbf_stack_sync_timeouts(const dbf_stack* S, int* timeouts) {
    if (!S) return DBF_EINVAL;
    return read_timeouts(S->plan, timeouts);
}

void dbf_stack_free(dbf_stack* S) {
    if (!S) return;
    free_plan(S->plan);
    std::free(S->h_x_prefix);
    std::free(S->h_y_prefix);
    delete S;
}

int dbf_tuning_set(int knob, int value) {
    if (knob < 0 || knob >= DBF_TUNE_COUNT_) return DBF_EINVAL;
    if (value < g_knobs[knob].lo || value > g_knobs[knob].hi) return DBF_EINVAL;
    g_knobs[knob].value = value;
    return DBF_OK;
}

int dbf_tuning_get(int knob) {
    if (knob < 0 || knob >= DBF_TUNE_COUNT_) return INT_MIN;
    return g_knobs[knob].value;
}

void dbf_tuning_reset(void) {
    for (Knob& k : g_knobs) k.value = k.def;
}

const char* dbf_strerror(int code) {
    switch (code) {
        case DBF_OK: return "ok";
        case DBF_EINVAL: return "invalid argument (null pointer, bad enum, batch or T out of range)";
        case DBF_ESHAPE: return "bad shape (n_in, n_out, k must be in [1, 2^20])";
        case DBF_ENOTSIGN: return "sign entry other than -1/+1, or non-zero tail bits";
        case DBF_ENOMEM: return "out of memory";
        case DBF_EHIP: return "HIP runtime error (no usable GPU, failed copy or launch)";
        case DBF_EWORKSPACE: return "workspace missing, misaligned or too small";
        default: return "unknown error code";
    }
}

}  // extern "C"

int dbf_tune(int knob) { return g_knobs[knob].value; }
