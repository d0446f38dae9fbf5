// Internal declarations shared by the host API and the HIP kernels of libdbf.
#ifndef DBF_INTERNAL_H
#define DBF_INTERNAL_H

#include "../../include/dbf.h"

#define DBF_TILE_ROWS 128
#define DBF_TILE_COLS 64
#define DBF_TILE_BYTES 1024
#define DBF_MAX_SPAN 16  /* most row tiles one workgroup takes */
#define DBF_SYNC_STRIDE 64  /* 64-bit words between the per-layer counters of a plan (DbfPlan::d_sync): 512 bytes, so
                              that polls of different counters spread over the memory channels */
#define DBF_PIECES_MAX_BATCH 2  /* largest batch for which row tiles may be cut into column pieces */
#define DBF_PIECE_CNT_STRIDE 32 /* ints between the arrival counters of two row tiles: 128 bytes, a cache line each (side by side
                                   the finishing atomics of a launch's workgroups queued at one line: a 4096 x 11008 layer
                                   alone 18.1 -> 17.0 us, 4096 x 14336 19.2 -> 18.0) */

static inline int dbf_row_tiles(int rows) { return (rows + DBF_TILE_ROWS - 1) / DBF_TILE_ROWS; }
static inline int dbf_col_tiles(int cols) { return (cols + DBF_TILE_COLS - 1) / DBF_TILE_COLS; }

// One sign-matrix stage of one layer as the vector-ALU kernel sees it (device memory).
//   B stage: bits = B tiled (k rows, n_in cols), in_scale = b, row_scale = m, input is the
//            caller's fp16 x, output is the layer's fp32 middle scratch t.
//   A stage: bits = A tiled (n_out rows, k cols), in_scale = NULL, row_scale = a, input is t,
//            output is the caller's fp16 y.
struct DbfStage {
    const uint8_t* bits;        // tiled signs, n_rt * n_ct tiles of 1 KiB
    const uint16_t* in_scale;   // fp16 [n_ct*64], zero padded, or NULL
    const uint16_t* row_scale;  // fp16 [n_rt*128], zero padded
    float* t;                   // fp32 [DBF_MAX_BATCH][t_stride] middle scratch of the layer
    long long x_off;            // element offset of this layer's x block, per unit of batch
    long long y_off;            // element offset of this layer's y block, per unit of batch
    int n_rt, n_ct;             // tiles along rows / cols
    int rows, cols;             // valid rows / cols
    int t_stride;               // elements between batch rows of t
    int pad_;
    unsigned char* q_in;        // the stage's input quantised once per call (batches of 2 and more, long-rows
                                // plans): float scale[16], int sigma[16], then int8 [n_ct][2 * batch][64]: per
                                // column tile the 64 bytes of plane 0, of plane 1, ... (plane 2 bi = high bytes,
                                // 2 bi + 1 = low bytes of batch row bi); room for 2 * 16 planes
};

// Work item of the vector-ALU kernel: one 128-row tile of one layer.
struct DbfWorkItem {
    int layer;
    int rt0;
    int nrt;
    int pad_;
};

// Work item of the matrix-core kernel: `nrt` consecutive row tiles of one stage of one layer,
// with everything the workgroup needs in one 120-byte record (scalar loads, no second hop
// through a per-layer table).  A launch list holds all B-stage items first, then all A-stage
// items, so that a fused launch dispatches every producer before any consumer.
struct DbfItem {
    const uint8_t* bits;        // first tile of the item's first row tile
    const uint16_t* in_scale;   // B stage: b (fp16, zero padded to n_ct*64); A stage: NULL
    const uint16_t* row_scale;  // fp16 scales starting at the item's first row (zero padded)
    float* t;                   // the layer's middle activations [DBF_MAX_BATCH][t_stride]
    long long io_off;           // B: element offset of the layer's x block, A: of its y block
                                // (both per unit of batch)
    int n_ct;                   // column tiles of the stage
    int nrt;                    // row tiles of this item (1..DBF_MAX_SPAN)
    int row0;                   // first row of the item
    int rows;                   // valid rows of the stage
    int cols;                   // valid columns of the stage
    int t_stride;               // elements between batch rows of t
    int layer;                  // index of the layer's counters (DbfPlan::d_sync)
    int need;                   // B-stage row tiles of the layer: what one launch adds to the "published" counter
    int stage_a;                // 0: B stage, 1: A stage
    int peers;                  // A-stage row tiles of the layer: what one launch adds to the "finished" counter
    // Column pieces (lists with pieces > 1 hold one row tile per item): the item covers column tiles
    // [ct0, ct0 + ct_n) of its row tile; the pieces of a row tile add their exact integer sums into
    // acc and the last one to arrive (cnt) scales and stores the result, and clears both.
    int ct0, ct_n;              // column tiles of this item (0, n_ct if the row tile is not cut)
    int pieces;                 // items that share this row tile (1: not cut)
    int acc_stride;             // elements between batch rows of acc
    int* acc;                   // int32 [DBF_PIECES_MAX_BATCH][acc_stride], this row tile's first row
    int* cnt;                   // arrival counter of this row tile (low 16 bits: pieces arrived; bit 16 and up:
                                // pieces that gave up their wait, so that the finishing piece knows)
    const unsigned char* q_in;  // the stage's quantised input (see DbfStage)
};
#define DBF_QIN_HEADER 128      /* bytes of scale[16] + sigma[16] in front of the planes */

// Device-side state of one launch plan: everything a decode call of a layer or a stack needs.
struct DbfPlan {
    void* dev_block;            // single allocation holding all tables below
    int n_layers;
    DbfStage* d_stagesB;        // [n_layers]
    DbfStage* d_stagesA;        // [n_layers]
    DbfWorkItem* d_workB1;      // vector-ALU work lists, one row tile per workgroup
    DbfWorkItem* d_workA1;
    int blocksB1, blocksA1;
    DbfItem* d_items_n;         // matrix-core items, up to `span` row tiles each: B items, then A items
    int nBn, nAn;
    DbfItem* d_items_s;         // the same with the row tiles per item chosen for the launches of batches of 2 and
    int nBs, nAs;               // more, which take a stage input quantised once per call (fewer, longer items)
    DbfItem* d_items_1;         // the same with one row tile per item (used when the columns of
    int nB1, nA1;               // a stage do not fit one LDS chunk at the requested batch)
    DbfItem* d_items_p;         // one row tile per item, row tiles cut into column pieces: built for plans
    int nBp, nAp;               // with few row tiles (a layer alone, a short stack); NULL otherwise
    int piece_row_tiles;        // row tiles of the larger stage over all layers (batch 2 takes d_items_p only for few)
    int rows_ok;                // the items of d_items_s are long enough to give each wavefront a row tile of its own
    int long_rows;              // stage inputs are quantised once per call at every batch (see build_plan)
    int x_vec_ok;               // every layer's x row at batch 1 starts at a multiple of 8 values and has a multiple of 8 columns
    // Counters of the one-launch kernel, 64 bits each, zero when the plan is built and only ever growing
    // (nothing is reset, so a workgroup that gives up its wait leaves them consistent):
    //   [layer]            B-stage row tiles published so far, over all launches of this plan
    //   [n_layers + layer] A-stage row tiles finished so far: divided by the layer's A row tiles this is
    //                      the number of completed launches, i.e. how much of the first counter is old
    // (what a launch adds is the same whichever of the plan's lists it uses)
    //   [2 n_layers]       waits given up (sticky)
    // (indices in units of DBF_SYNC_STRIDE words: each counter has 512 bytes to itself)
    unsigned long long* d_sync;
    int span;                   // row tiles per item in d_items_n
    int max_cols_B, max_cols_A;
};

struct dbf_layer {
    int n_in, n_out, k;
    int device;
    void* dev_block;        // the single device allocation everything below points into
    size_t device_bytes;
    uint8_t* dA;            // tiled A: rows n_out, cols k
    uint8_t* dB;            // tiled B: rows k, cols n_in
    uint16_t* da;           // fp16 [row_tiles(n_out)*128]
    uint16_t* dm;           // fp16 [row_tiles(k)*128]
    uint16_t* db;           // fp16 [col_tiles(n_in)*64]
    float* dt;              // fp32 [DBF_MAX_BATCH][t_stride]
    int t_stride;
    unsigned char* dqB;     // quantised input of the B stage (DbfStage::q_in)
    unsigned char* dqA;     // quantised input of the A stage
    DbfStage h_stages[2];   // {B stage, A stage} with offsets 0
    DbfPlan plan;           // launch plan of this layer alone
};

// Tuning and test hooks (dbf_tuning_set); index = DBF_TUNE_*.
int dbf_tune(int knob);

struct dbf_stack {
    int n_layers;
    int device;
    DbfPlan plan;
    long long* h_x_prefix;  // host [n_layers+1] prefix sums of n_in
    long long* h_y_prefix;  // host [n_layers+1] prefix sums of n_out
};

#endif  // DBF_INTERNAL_H
