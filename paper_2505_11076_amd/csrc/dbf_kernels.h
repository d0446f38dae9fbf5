// Launchers of the HIP kernels (defined in the .hip files, called from dbf_api.hip).
#ifndef DBF_KERNELS_H
#define DBF_KERNELS_H

#include <hip/hip_runtime.h>

#include "dbf_internal.h"

// One stage (B or A): `blocks` workgroups, workgroup i handles work[i].  x_base / y_base are
// the caller's fp16 buffers (only the one the stage touches is used).  max_cols = largest
// `cols` over the table (sizes the LDS staging).  The VALU kernel takes items with nrt == 1
// only; the MFMA kernel takes nrt > 1 only when all columns fit one LDS chunk, i.e. when
// dbf_mfma_chunk_tiles(batch, max_cols) covers every layer's column tiles.
hipError_t dbf_launch_stage_valu(bool stage_a, const DbfStage* table, const DbfWorkItem* work,
                                 int blocks, const void* x_base, void* y_base, int batch,
                                 int max_cols, hipStream_t stream);
hipError_t dbf_launch_stage_mfma(bool stage_a, const DbfStage* table, const DbfWorkItem* work,
                                 int blocks, const void* x_base, void* y_base, int batch,
                                 int max_cols, hipStream_t stream);
int dbf_mfma_chunk_tiles(int batch, int max_cols);

#endif  // DBF_KERNELS_H
