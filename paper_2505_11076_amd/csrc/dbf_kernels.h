// Launchers of the HIP kernels (defined in the .hip files, called from dbf_api.hip).
#ifndef DBF_KERNELS_H
#define DBF_KERNELS_H

#include <hip/hip_runtime.h>

#include "dbf_internal.h"

// Vector-ALU kernel, one stage (B or A): `blocks` workgroups, workgroup i handles work[i]
// (one row tile).  x_base / y_base are the caller's fp16 buffers (only the one the stage
// touches is used).
hipError_t dbf_launch_stage_valu(bool stage_a, const DbfStage* table, const DbfWorkItem* work,
                                 int blocks, const void* x_base, void* y_base, int batch,
                                 hipStream_t stream);

// Matrix-core kernel over items[0..n_items): workgroup i handles items[i].
//   use_sync != 0 (fused launch of B items followed by A items): an A-stage workgroup waits, for at most
//   wait_limit_us microseconds, until the layer's B-stage workgroups of THIS launch have published all their
//   rows (sync, see DbfPlan::d_sync); a workgroup that gives up writes NaN outputs and counts a time-out.
//   use_sync == 0: no waiting and no counters (the caller orders the stages by launches).
// Items with nrt > 1 are allowed only if every item's columns fit one LDS chunk, i.e.
// dbf_mfma_chunk_tiles(batch, max_cols, shared_q) >= dbf_col_tiles(max_cols).
//   pieces != 0: the list may hold column pieces of row tiles (DbfItem::pieces > 1; one row tile per
//   item, batch <= DBF_PIECES_MAX_BATCH); pieces == 0: every item covers all columns of its row tiles.
//   shared_q != 0: the input of the items' stage has been quantised for the whole launch by
//   dbf_launch_quantise_inputs (same stream, earlier); the items copy it instead of quantising it themselves.
//   Only with use_sync == 0 and pieces == 0.
//   one_pass_rows != 0: the caller has checked that every B-stage row of the launch can be read in 16-byte pieces
//   (columns a multiple of 8, 16-byte aligned address at this batch), so that at batch 1 rows of up to
//   dbf_mfma_one_pass_cols() columns all take the one-pass prologue -- which the fp4 x bf6 form of the kernel needs.
hipError_t dbf_launch_items_mfma(const DbfItem* items, int n_items, unsigned long long* sync, int n_layers,
                                 int use_sync, const void* x_base, void* y_base, int batch,
                                 int max_cols, int pieces, int shared_q, int one_pass_rows, int wait_limit_us,
                                 hipStream_t stream);
// Quantises the input of one stage (stage_a = 0: x times b of every layer, 1: the middle activations) of the
// n_layers stages in d_stages for `batch` rows into the stages' q_in buffers.
hipError_t dbf_launch_quantise_inputs(const DbfStage* d_stages, int n_layers, int stage_a, const void* x_base,
                                      int batch, hipStream_t stream);
int dbf_mfma_chunk_tiles(int batch, int max_cols, int shared_q);
// Widest input row (columns) the matrix-core kernel's one-pass prologue takes at batch 1: such rows are
// read once and quantised from registers; wider ones are read twice (scale, then quantisation).
int dbf_mfma_one_pass_cols();
// One-time, per-process set-up of the matrix-core decode kernels (LDS limits); cheap to call again.
hipError_t dbf_mfma_prepare();

// Prefill (T tokens): two stages with the middle activations in the caller's workspace; arguments are
// validated by dbf_gemm before this is called.  int8 matrix cores as the adder (masked sign bytes as one
// operand, the activations rounded per token to 16-bit fixed point and split into two int8 planes), exact
// integer sums, middle activations in fp32.
struct dbf_layer;
// (calls of few tokens cut the columns of a stage into shares over more workgroups; the integer sums they add up
//  need room of their own, which _bytes counts and _bytes_without_splits does not: the launcher splits only where
//  workspace_bytes covers it)
size_t dbf_gemm_i8_workspace_bytes(const dbf_layer* L, int T);
size_t dbf_gemm_i8_workspace_bytes_without_splits(const dbf_layer* L, int T);
hipError_t dbf_gemm_i8_launch(const dbf_layer* L, const void* X_dev, void* Y_dev, int T, void* workspace_dev,
                              size_t workspace_bytes, hipStream_t stream);

// Middle-channel pruning: fills the sign tiles and vectors of `dst` (a freshly created layer with
// k = n_keep on the same device) from `src` and the kept middle indices keep_dev (device, increasing,
// each < src->k).  Queued on `stream`.
hipError_t dbf_prune_launch(const dbf_layer* src, dbf_layer* dst, const int* keep_dev, int n_keep, hipStream_t stream);

#endif  // DBF_KERNELS_H
