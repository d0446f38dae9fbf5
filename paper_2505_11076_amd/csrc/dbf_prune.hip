// Middle-channel pruning in the tiled layout (paper, section 3.5: the middle dimension is treated as
// channels and only some are kept; choosing them needs gradients and is the caller's business).
// Given the kept middle indices keep[0..k') (increasing), the new layer has
//     A'[:, j'] = A[:, keep[j']],   B'[j', :] = B[keep[j'], :],   m'[j'] = m[keep[j']],
// a and b unchanged.  Both sign matrices stay in the device tile layout (tile = 128 rows x 64
// columns = 1 KiB, byte 256 g + 16 r + j, bit s = sign(row 16 s + r, column 16 g + j)):
//   * a COLUMN of a tile is one byte position in each of its 16 r-rows, all eight bit planes at
//     once, so the column gather of A is a byte gather;
//   * a ROW of a tile is one bit plane of one r-row, so the row gather of B takes bit s_o of the
//     64 bytes of the old row and deposits it as bit s of the new row's bytes; the eight rows that
//     share an output byte are combined by OR in LDS.
// Every output tile is written whole (padding rows / columns as zero bits), one workgroup per tile,
// coalesced 4-byte stores.  Bandwidth bound: reads about the kept part of the old signs, writes the new.
#include "dbf_kernels.h"

namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

// A': out tile (rt, ct') <- bytes of old tiles (rt, keep[.] / 64).  256 threads: thread -> new column
// ci = tid / 4 of the tile and four of its sixteen r-rows.
__global__ __launch_bounds__(256) void dbf_prune_cols_kernel(const uint8_t* __restrict__ old_bits, int old_n_ct,
                                                            uint8_t* __restrict__ new_bits, int new_n_ct,
                                                            const int* __restrict__ keep, int n_keep) {
    __shared__ __align__(16) uint8_t tile[DBF_TILE_BYTES];
    const int rt = blockIdx.y, ctn = blockIdx.x, tid = threadIdx.x;
    const int ci = tid >> 2, q = tid & 3;
    const int cn = ctn * DBF_TILE_COLS + ci;                 // new column
    const int gn = ci >> 4, jn = ci & 15;
    if (cn < n_keep) {
        const int o = keep[cn];
        const uint8_t* src = old_bits + ((size_t)rt * old_n_ct + (o >> 6)) * DBF_TILE_BYTES + 256 * ((o & 63) >> 4) + (o & 15);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int r = 4 * q + i;
            tile[256 * gn + 16 * r + jn] = src[16 * r];
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) tile[256 * gn + 16 * (4 * q + i) + jn] = 0;
    }
    __syncthreads();
    reinterpret_cast<unsigned*>(new_bits + ((size_t)rt * new_n_ct + ctn) * DBF_TILE_BYTES)[tid] =
        reinterpret_cast<const unsigned*>(tile)[tid];
}

// B': out tile (rt', ct) <- bit planes of old tiles (keep[.] / 128, ct).  256 threads: thread -> new row
// rho = tid / 2 of the tile (bit s = rho / 16 of r-row rho % 16) and two of the four column groups.
__global__ __launch_bounds__(256) void dbf_prune_rows_kernel(const uint8_t* __restrict__ old_bits,
                                                            uint8_t* __restrict__ new_bits, int n_ct,
                                                            const int* __restrict__ keep, int n_keep) {
    __shared__ __align__(16) unsigned tile[DBF_TILE_BYTES / 4];
    const int rtn = blockIdx.y, ct = blockIdx.x, tid = threadIdx.x;
    tile[tid] = 0;
    __syncthreads();
    const int rho = tid >> 1, hf = tid & 1;
    const int s = rho >> 4, r = rho & 15;
    const int rn = rtn * DBF_TILE_ROWS + rho;                // new row
    if (rn < n_keep) {
        const int o = keep[rn];
        const int so = (o & 127) >> 4, ro = o & 15;
        const uint8_t* src = old_bits + ((size_t)(o >> 7) * n_ct + ct) * DBF_TILE_BYTES + 16 * ro;
#pragma unroll
        for (int gi = 0; gi < 2; ++gi) {
            const int g = 2 * hf + gi;
            const v4u w = *reinterpret_cast<const v4u*>(src + 256 * g);
            unsigned* dst = tile + (256 * g + 16 * r) / 4;
            atomicOr(dst + 0, ((w.x >> so) & 0x01010101u) << s);
            atomicOr(dst + 1, ((w.y >> so) & 0x01010101u) << s);
            atomicOr(dst + 2, ((w.z >> so) & 0x01010101u) << s);
            atomicOr(dst + 3, ((w.w >> so) & 0x01010101u) << s);
        }
    }
    __syncthreads();
    reinterpret_cast<unsigned*>(new_bits + ((size_t)rtn * n_ct + ct) * DBF_TILE_BYTES)[tid] = tile[tid];
}

// m'[i] = m[keep[i]], zero beyond the kept channels (the vector is padded to whole row tiles).
__global__ void dbf_prune_scale_kernel(const uint16_t* __restrict__ old_m, uint16_t* __restrict__ new_m,
                                       const int* __restrict__ keep, int n_keep, int padded) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < padded) new_m[i] = i < n_keep ? old_m[keep[i]] : (uint16_t)0;
}

}  // namespace

// src: the layer to prune; dst: a freshly created layer with k = n_keep (its buffers allocated, vectors
// zeroed); keep_dev: device copy of the kept indices.  Everything is queued on `stream`.
hipError_t dbf_prune_launch(const dbf_layer* src, dbf_layer* dst, const int* keep_dev, int n_keep, hipStream_t stream) {
    const int rtA = dbf_row_tiles(src->n_out), ctA_old = dbf_col_tiles(src->k), ctA_new = dbf_col_tiles(n_keep);
    const int rtB_new = dbf_row_tiles(n_keep), ctB = dbf_col_tiles(src->n_in);
    hipLaunchKernelGGL(dbf_prune_cols_kernel, dim3(ctA_new, rtA), dim3(256), 0, stream, src->dA, ctA_old, dst->dA,
                       ctA_new, keep_dev, n_keep);
    hipLaunchKernelGGL(dbf_prune_rows_kernel, dim3(ctB, rtB_new), dim3(256), 0, stream, src->dB, dst->dB, ctB, keep_dev,
                       n_keep);
    const int padded = rtB_new * DBF_TILE_ROWS;
    hipLaunchKernelGGL(dbf_prune_scale_kernel, dim3((padded + 255) / 256), dim3(256), 0, stream, src->dm, dst->dm,
                       keep_dev, n_keep, padded);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    e = hipMemcpyAsync(dst->da, src->da, 2 * (size_t)rtA * DBF_TILE_ROWS, hipMemcpyDeviceToDevice, stream);
    if (e != hipSuccess) return e;
    return hipMemcpyAsync(dst->db, src->db, 2 * (size_t)ctB * DBF_TILE_COLS, hipMemcpyDeviceToDevice, stream);
}
