// Launchers of the HIP kernels (defined in the .hip files, called from dbf_api.hip).
#ifndef DBF_KERNELS_H
#define DBF_KERNELS_H

#include <hip/hip_runtime.h>

#include "dbf_internal.h"

// One stage (B or A) of `blocks` (layer, row-tile) work items.  `map` may be NULL for a
// single layer (work item i = row tile i of table[0]).  x_base / y_base are the caller's
// fp16 buffers (only the one the stage touches is used).  max_cols = largest `cols` over
// the table (sizes the LDS staging).
hipError_t dbf_launch_stage_valu(bool stage_a, const DbfStage* table, const DbfBlockRef* map,
                                 int blocks, const void* x_base, void* y_base, int batch,
                                 int max_cols, hipStream_t stream);
hipError_t dbf_launch_stage_mfma(bool stage_a, const DbfStage* table, const DbfBlockRef* map,
                                 int blocks, const void* x_base, void* y_base, int batch,
                                 int max_cols, hipStream_t stream);

#endif  // DBF_KERNELS_H
