// Decode stage with the int8 matrix cores as the adder.
//
// One sign-matrix product of the forward-pass expression (paper, section 3):
//     out[row] = row_scale[row] * sum_col S[row][col] * u[col],
// u = x . b (B stage) or u = t (A stage).  Inside the product only additions are needed
// (section 3.1, "Inference costs"); at one vector-ALU add per sign bit, however, the ALU and
// not HBM would bound the kernel on this chip (64 lane-operations per clock per CU against
// ~104 sign bits per clock per CU at 8 TB/s).  So the additions are done by
// v_mfma_i32_16x16x64_i8 instead:
//
//   * u is rounded once to 16-bit fixed point, q = rint(u * 32512 / max|u|) (per batch row),
//     and split into two int8 pieces q = 256*hi + lo.  Integer sums are exact, so the only
//     error of the stage is this rounding (about 4e-5 of rms(u) for Gaussian inputs).
//   * A lane's 16-byte load of a tile holds 16 columns; bit s of each byte belongs to row
//     group s.  (bytes & (0x01010101 << s)) is directly the A operand (16 rows x 64 cols of
//     values 0 or 2^s, -128 for s = 7) of one matrix instruction: one AND per four signs.
//   * The B operand holds the pieces of u in columns 2*bi (hi) and 2*bi+1 (lo) for batch row
//     bi, so up to 8 batch rows ride in one instruction (16 with two column groups).
//   * acc_s = 2^s * sum_{bit=1} q.  With sigma = sum_col q, the signed sum is
//     2 * (acc_s >> s) - sigma, exactly, in int32.
//
// Work split: one workgroup (4 wavefronts) per 128-row tile; wavefront w walks column tiles
// w, w+4, ...; the four partial results are added with integer LDS atomics (order does not
// matter for integers, so the result is deterministic).
#include "dbf_kernels.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));

constexpr int PF = 4;              // tiles of sign bits kept in flight per wavefront
constexpr float QMAX = 32512.f;    // 127*256: largest |q| so that hi and lo fit int8
constexpr int XQ_PAD = 16;         // bytes of padding per operand row (LDS bank spread)

__device__ inline float half_bits_to_float(uint16_t h) {
    return (float)__builtin_bit_cast(_Float16, h);
}
__device__ inline uint16_t float_to_half_bits(float f) {
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}

__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}
__device__ inline int wave_sum(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}

template <bool STAGE_A>
__device__ inline float load_u(const DbfStage& st, const uint16_t* x, int bi, int l) {
    if (STAGE_A) return st.t[(size_t)bi * st.t_stride + l];
    return half_bits_to_float(x[(size_t)bi * st.cols + l]) * half_bits_to_float(st.in_scale[l]);
}

// LDS carve-up (dynamic): red | misc | xq
struct Misc {
    float scale[DBF_MAX_BATCH];   // u ~= q * scale
    float inv[DBF_MAX_BATCH];     // q = rint(u * inv)
    int sigma[DBF_MAX_BATCH];     // sum over all columns of q
    float wmax[4][DBF_MAX_BATCH]; // per-wavefront max|u|
};

template <bool STAGE_A, int NCG>
__global__ __launch_bounds__(256) void dbf_stage_mfma_kernel(const DbfStage* __restrict__ table,
                                                             const DbfBlockRef* __restrict__ map,
                                                             const uint16_t* __restrict__ x_base,
                                                             uint16_t* __restrict__ y_base,
                                                             int batch, int ch_tiles) {
    extern __shared__ __align__(16) unsigned char smem[];
    int* red = reinterpret_cast<int*>(smem);                                   // [NCG][8][64][4]
    Misc* misc = reinterpret_cast<Misc*>(smem + NCG * 8192);
    signed char* xq = reinterpret_cast<signed char*>(smem + NCG * 8192 + 512);  // [ncols][chs]

    int layer = 0, rt = blockIdx.x;
    if (map) {
        layer = map[blockIdx.x].layer;
        rt = map[blockIdx.x].rt;
    }
    const DbfStage st = table[layer];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int g = lane >> 4, c = lane & 15;
    const int ncols = 2 * batch;
    const int chs = ch_tiles * DBF_TILE_COLS + XQ_PAD;
    const uint4* tiles = reinterpret_cast<const uint4*>(st.bits) + (size_t)rt * st.n_ct * 64 + lane;
    const uint16_t* x = x_base + st.x_off * batch;
    uint16_t* y = y_base + st.y_off * batch;

    // ---- per batch row: max|u|, then the fixed-point scale -------------------------------
    for (int bi = 0; bi < batch; ++bi) {
        float mx = 0.f;
        for (int l = tid; l < st.cols; l += 256) mx = fmaxf(mx, fabsf(load_u<STAGE_A>(st, x, bi, l)));
        mx = wave_max(mx);
        if (lane == 0) misc->wmax[w][bi] = mx;
    }
    for (int i = tid; i < NCG * 2048; i += 256) red[i] = 0;
    __syncthreads();
    if (tid < batch) {
        const float mx = fmaxf(fmaxf(misc->wmax[0][tid], misc->wmax[1][tid]),
                               fmaxf(misc->wmax[2][tid], misc->wmax[3][tid]));
        misc->scale[tid] = mx / QMAX;
        misc->inv[tid] = mx > 0.f ? QMAX / mx : 0.f;
        misc->sigma[tid] = 0;
    }
    __syncthreads();

    v4i acc[NCG][8];
#pragma unroll
    for (int gi = 0; gi < NCG; ++gi)
#pragma unroll
        for (int s = 0; s < 8; ++s) acc[gi][s] = (v4i){0, 0, 0, 0};

    // operand row this lane feeds to the matrix instruction (unused columns alias a valid row)
    int xrow[NCG];
#pragma unroll
    for (int gi = 0; gi < NCG; ++gi) {
        const int col = 16 * gi + c;
        xrow[gi] = (col < ncols ? col : col % ncols) * chs + 16 * g;
    }

    for (int c0 = 0; c0 < st.n_ct; c0 += ch_tiles) {
        const int cend = min(st.n_ct, c0 + ch_tiles);
        if (c0 > 0) __syncthreads();  // everyone is done reading the previous chunk
        // ---- quantise columns [64*c0, 64*cend) of every batch row into LDS ----------------
        for (int bi = 0; bi < batch; ++bi) {
            const float inv = misc->inv[bi];
            int local = 0;
            signed char* hi_row = xq + (2 * bi) * chs;
            signed char* lo_row = xq + (2 * bi + 1) * chs;
            for (int l = c0 * 64 + tid; l < cend * 64; l += 256) {
                int q = 0;
                if (l < st.cols) {
                    float f = rintf(load_u<STAGE_A>(st, x, bi, l) * inv);
                    f = fminf(fmaxf(f, -QMAX), QMAX);
                    q = (int)f;
                }
                const int lo = ((q + 128) & 255) - 128;
                const int hi = (q - lo) >> 8;
                hi_row[l - c0 * 64] = (signed char)hi;
                lo_row[l - c0 * 64] = (signed char)lo;
                local += q;
            }
            local = wave_sum(local);
            if (lane == 0) atomicAdd(&misc->sigma[bi], local);
        }
        __syncthreads();

        // ---- stream this wavefront's tiles of the chunk ------------------------------------
        const int first = c0 + w;
        const int nt = (cend - first + 3) >> 2;  // tiles first, first+4, ... < cend
        uint4 buf[PF];
#pragma unroll
        for (int i = 0; i < PF; ++i)
            if (i < nt) buf[i] = tiles[(size_t)(first + 4 * i) * 64];
        for (int i0 = 0; i0 < nt; i0 += PF) {
#pragma unroll
            for (int i = 0; i < PF; ++i) {
                if (i0 + i < nt) {
                    const uint4 cur = buf[i];
                    if (i0 + i + PF < nt) buf[i] = tiles[(size_t)(first + 4 * (i0 + i + PF)) * 64];
                    const int xo = (first + 4 * (i0 + i) - c0) * 64;
                    v4i xop[NCG];
#pragma unroll
                    for (int gi = 0; gi < NCG; ++gi)
                        xop[gi] = *reinterpret_cast<const v4i*>(xq + xrow[gi] + xo);
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        const uint32_t msk = 0x01010101u << s;
                        v4i a;
                        a.x = (int)(cur.x & msk);
                        a.y = (int)(cur.y & msk);
                        a.z = (int)(cur.z & msk);
                        a.w = (int)(cur.w & msk);
#pragma unroll
                        for (int gi = 0; gi < NCG; ++gi)
                            acc[gi][s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, xop[gi], acc[gi][s], 0, 0, 0);
                    }
                }
            }
        }
    }

    // ---- combine the four wavefronts (integer adds: exact and order independent) ---------
#pragma unroll
    for (int gi = 0; gi < NCG; ++gi) {
        if (16 * gi + c < ncols) {
#pragma unroll
            for (int s = 0; s < 8; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i) atomicAdd(&red[((gi * 8 + s) * 64 + lane) * 4 + i], acc[gi][s][i]);
        }
    }
    __syncthreads();

    // ---- epilogue: result element (row 4*g'+i of group s, column) sits in lane 16*g'+column
    const int rho = tid & 127;
    const int s = rho >> 4, g2 = (rho & 15) >> 2, i2 = rho & 3;
    const int row = rt * DBF_TILE_ROWS + rho;
    const float rscale = half_bits_to_float(st.row_scale[row]);
    for (int bi = tid >> 7; bi < batch; bi += 2) {
        const int col = 2 * bi;
        const int gi = col >> 4, cc = col & 15;
        int vh = red[((gi * 8 + s) * 64 + 16 * g2 + cc) * 4 + i2];
        int vl = red[((gi * 8 + s) * 64 + 16 * g2 + cc + 1) * 4 + i2];
        if (s < 7) {
            vh >>= s;
            vl >>= s;
        } else {
            vh = -(vh >> 7);
            vl = -(vl >> 7);
        }
        const int total = 2 * (vh * 256 + vl) - misc->sigma[bi];
        const float val = (float)total * misc->scale[bi] * rscale;
        if (STAGE_A) {
            if (row < st.rows) y[(size_t)bi * st.rows + row] = float_to_half_bits(val);
        } else {
            st.t[(size_t)bi * st.t_stride + row] = val;  // padded rows have scale 0
        }
    }
}

}  // namespace

hipError_t dbf_launch_stage_mfma(bool stage_a, const DbfStage* table, const DbfBlockRef* map,
                                 int blocks, const void* x_base, void* y_base, int batch,
                                 int max_cols, hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    const uint16_t* x = static_cast<const uint16_t*>(x_base);
    uint16_t* y = static_cast<uint16_t*>(y_base);
    const int ncg = batch > 8 ? 2 : 1;
    const int ncols = 2 * batch;
    const int budget = ncg == 2 ? 40960 : 32768;  // LDS bytes for the quantised operand
    int ch_tiles = ((budget / ncols - XQ_PAD) / DBF_TILE_COLS) & ~3;
    const int need = (dbf_col_tiles(max_cols) + 3) & ~3;
    if (ch_tiles > need) ch_tiles = need;
    if (ch_tiles < 4) ch_tiles = 4;
    const size_t smem = (size_t)ncg * 8192 + 512 + (size_t)ncols * (ch_tiles * DBF_TILE_COLS + XQ_PAD);
    if (ncg == 1) {
        if (stage_a)
            hipLaunchKernelGGL((dbf_stage_mfma_kernel<true, 1>), dim3(blocks), dim3(256), smem, stream,
                               table, map, x, y, batch, ch_tiles);
        else
            hipLaunchKernelGGL((dbf_stage_mfma_kernel<false, 1>), dim3(blocks), dim3(256), smem, stream,
                               table, map, x, y, batch, ch_tiles);
    } else {
        if (stage_a)
            hipLaunchKernelGGL((dbf_stage_mfma_kernel<true, 2>), dim3(blocks), dim3(256), smem, stream,
                               table, map, x, y, batch, ch_tiles);
        else
            hipLaunchKernelGGL((dbf_stage_mfma_kernel<false, 2>), dim3(blocks), dim3(256), smem, stream,
                               table, map, x, y, batch, ch_tiles);
    }
    return hipGetLastError();
}
