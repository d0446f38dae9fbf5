// Decode stage on the vector ALU: one fp32 add or subtract per sign bit.
//
// This is the plain evaluation of one sign-matrix product of the forward-pass expression
// (paper, section 3): out[row] = row_scale[row] * sum_col S[row][col] * u[col], where
// u = x . b for the B stage and u = t for the A stage, and S is read from the tiled bit
// layout.  It keeps exact fp32 sums and serves as the reference variant on the GPU; the
// matrix-core variant is the fast one.
//
// Work split: one workgroup (4 wavefronts) per 128-row tile.  The input vector of one batch
// row is staged in LDS as fp32; wavefront w walks column tiles w, w+4, ...; a lane loads its
// 16 bytes of the tile (16 columns x 8 row groups) and updates eight accumulators.  Partial
// sums are combined over the four 16-column lane groups by cross-lane shuffles and over the
// four wavefronts through LDS, always in the same order (deterministic).
#include "dbf_kernels.h"

namespace {

constexpr int VALU_CHUNK_TILES = 128;  // 128 tiles * 64 cols * 4 B = 32 KiB of staged input

__device__ inline float half_bits_to_float(uint16_t h) {
    return (float)__builtin_bit_cast(_Float16, h);
}

__device__ inline uint16_t float_to_half_bits(float f) {
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}

template <bool STAGE_A>
__global__ __launch_bounds__(256) void dbf_stage_valu_kernel(const DbfStage* __restrict__ table,
                                                             const DbfWorkItem* __restrict__ work,
                                                             const uint16_t* __restrict__ x_base,
                                                             uint16_t* __restrict__ y_base,
                                                             int batch) {
    __shared__ float su[VALU_CHUNK_TILES * DBF_TILE_COLS];
    __shared__ float red[4][DBF_TILE_ROWS];

    const int rt = work[blockIdx.x].rt0;  // items of this kernel span one row tile
    const DbfStage st = table[work[blockIdx.x].layer];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int g = lane >> 4, r = lane & 15;
    const uint4* tiles = reinterpret_cast<const uint4*>(st.bits) + (size_t)rt * st.n_ct * 64;
    const uint16_t* x = x_base + st.x_off * batch;
    uint16_t* y = y_base + st.y_off * batch;

    for (int bi = 0; bi < batch; ++bi) {
        float acc[8];
#pragma unroll
        for (int s = 0; s < 8; ++s) acc[s] = 0.f;

        for (int c0 = 0; c0 < st.n_ct; c0 += VALU_CHUNK_TILES) {
            const int cend = min(st.n_ct, c0 + VALU_CHUNK_TILES);
            __syncthreads();
            for (int l = c0 * 64 + tid; l < cend * 64; l += 256) {
                float u = 0.f;
                if (l < st.cols) {
                    if (STAGE_A)
                        u = st.t[(size_t)bi * st.t_stride + l];
                    else
                        u = half_bits_to_float(x[(size_t)bi * st.cols + l]) *
                            half_bits_to_float(st.in_scale[l]);
                }
                su[l - c0 * 64] = u;
            }
            __syncthreads();
            for (int ct = c0 + w; ct < cend; ct += 4) {
                const uint4 bits = tiles[(size_t)ct * 64 + lane];
                const float* up = su + (ct - c0) * 64 + 16 * g;
                const uint32_t words[4] = {bits.x, bits.y, bits.z, bits.w};
#pragma unroll
                for (int v = 0; v < 4; ++v) {
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float u = up[4 * v + q];
                        const uint32_t byte = words[v] >> (8 * q);
#pragma unroll
                        for (int s = 0; s < 8; ++s) acc[s] += ((byte >> s) & 1u) ? u : -u;
                    }
                }
            }
        }
        // combine the four 16-column lane groups (lanes r, r+16, r+32, r+48)
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            acc[s] += __shfl_xor(acc[s], 16);
            acc[s] += __shfl_xor(acc[s], 32);
        }
        __syncthreads();
        if (g == 0) {
#pragma unroll
            for (int s = 0; s < 8; ++s) red[w][16 * s + r] = acc[s];
        }
        __syncthreads();
        if (tid < DBF_TILE_ROWS) {
            const float sum = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
            const int row = rt * DBF_TILE_ROWS + tid;
            const float val = sum * half_bits_to_float(st.row_scale[row]);
            if (STAGE_A) {
                if (row < st.rows) y[(size_t)bi * st.rows + row] = float_to_half_bits(val);
            } else {
                st.t[(size_t)bi * st.t_stride + row] = val;  // padded rows have scale 0
            }
        }
    }
}

}  // namespace

hipError_t dbf_launch_stage_valu(bool stage_a, const DbfStage* table, const DbfWorkItem* work,
                                 int blocks, const void* x_base, void* y_base, int batch,
                                 hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    const uint16_t* x = static_cast<const uint16_t*>(x_base);
    uint16_t* y = static_cast<uint16_t*>(y_base);
    if (stage_a)
        hipLaunchKernelGGL(dbf_stage_valu_kernel<true>, dim3(blocks), dim3(256), 0, stream, table,
                           work, x, y, batch);
    else
        hipLaunchKernelGGL(dbf_stage_valu_kernel<false>, dim3(blocks), dim3(256), 0, stream, table,
                           work, x, y, batch);
    return hipGetLastError();
}
