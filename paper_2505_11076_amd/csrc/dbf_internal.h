// Internal declarations shared by the host API and the HIP kernels of libdbf.
#ifndef DBF_INTERNAL_H
#define DBF_INTERNAL_H

#include "../../include/dbf.h"

#define DBF_TILE_ROWS 128
#define DBF_TILE_COLS 64
#define DBF_TILE_BYTES 1024

static inline int dbf_row_tiles(int rows) { return (rows + DBF_TILE_ROWS - 1) / DBF_TILE_ROWS; }
static inline int dbf_col_tiles(int cols) { return (cols + DBF_TILE_COLS - 1) / DBF_TILE_COLS; }

// One sign-matrix stage of one layer as the kernels see it (lives in device memory).
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
};

// Work item of one workgroup: `nrt` consecutive 128-row tiles of one layer, starting at rt0.
struct DbfWorkItem {
    int layer;
    int rt0;
    int nrt;
    int pad_;
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
    DbfStage* d_stages;     // device copy of {B stage, A stage}
    DbfStage h_stages[2];   // host copy
    DbfWorkItem* d_workB;   // device [n_rt of B]: one row tile per workgroup
    DbfWorkItem* d_workA;   // device [n_rt of A]
};

struct dbf_stack {
    int n_layers;
    int device;
    void* dev_block;
    DbfStage* d_stagesB;    // device [n_layers]
    DbfStage* d_stagesA;    // device [n_layers]
    DbfWorkItem* d_workB1;  // device [blocksB1]: one row tile per workgroup
    DbfWorkItem* d_workA1;  // device [blocksA1]
    DbfWorkItem* d_workBn;  // device [blocksBn]: several row tiles per workgroup
    DbfWorkItem* d_workAn;  // device [blocksAn]
    int blocksB1, blocksA1, blocksBn, blocksAn;
    int max_ct_B, max_ct_A; // largest number of column tiles over the layers
    int max_cols_B, max_cols_A;
    long long* h_x_prefix;  // host [n_layers+1] prefix sums of n_in
    long long* h_y_prefix;  // host [n_layers+1] prefix sums of n_out
};

#endif  // DBF_INTERNAL_H
