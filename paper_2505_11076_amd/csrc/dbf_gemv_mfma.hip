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
// Work split: a workgroup (4 wavefronts) takes `nrt` consecutive 128-row tiles of one layer
// and quantises the input vector once for all of them.  Within a row tile wavefront w walks
// column tiles w, w+4, ... with PF tiles of sign bits in flight (buffer loads whose
// out-of-range lanes return zero, so the steady-state loop has no branches); the loads for
// the next row tile are already in flight while the current one is reduced.  The four
// partial results are added with integer LDS atomics (exact, order independent).
#include "dbf_kernels.h"

// 1: tile loads by inline assembly with exact hand-placed waits (the fast path).
// 0: the same loads through the compiler builtin (it then waits with vmcnt(0) per group).
#ifndef DBF_ASM_LOADS
#define DBF_ASM_LOADS 1
#endif

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned short us8 __attribute__((ext_vector_type(8)));

constexpr int PF = 8;              // tiles of sign bits kept in flight per wavefront
constexpr int UNR = 4;             // independent 16-byte loads per thread in the prologue
constexpr float QMAX = 32512.f;    // 127*256: largest |q| so that hi and lo fit int8
constexpr int XQ_PAD = 16;         // bytes of padding per operand row (LDS bank spread)
constexpr unsigned OOB = 0x80000000u;  // buffer offset that is out of range for any span

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

// LDS carve-up (dynamic): red | misc | xq
struct Misc {
    float scale[DBF_MAX_BATCH];   // u ~= q * scale
    float inv[DBF_MAX_BATCH];     // q = rint(u * inv)
    int sigma[DBF_MAX_BATCH];     // sum over all columns of q
    float wmax[4][DBF_MAX_BATCH]; // per-wavefront max|u|
};

// Eight consecutive input values u[8*v .. 8*v+7] of batch row bi (vector item v).
// B stage: x (fp16) times b (fp16), exact in fp32.  A stage: the fp32 middle activations.
template <bool STAGE_A>
struct InputVec {
    v4u r0, r1;
    __device__ inline void load(const DbfStage& st, const uint16_t* x, int bi, int v, bool x_ok) {
        if (STAGE_A) {
            const v4f* p = reinterpret_cast<const v4f*>(st.t + (size_t)bi * st.t_stride) + 2 * (size_t)v;
            r0 = __builtin_bit_cast(v4u, p[0]);
            r1 = __builtin_bit_cast(v4u, p[1]);
        } else {
            r1 = __builtin_bit_cast(v4u, reinterpret_cast<const us8*>(st.in_scale)[v]);
            r0 = (v4u){0, 0, 0, 0};
            if (x_ok) r0 = __builtin_bit_cast(v4u, reinterpret_cast<const us8*>(x + (size_t)bi * st.cols)[v]);
        }
    }
    __device__ inline void get(float (&u)[8]) const {
        if (STAGE_A) {
            const v4f f0 = __builtin_bit_cast(v4f, r0), f1 = __builtin_bit_cast(v4f, r1);
            u[0] = f0.x;  u[1] = f0.y;  u[2] = f0.z;  u[3] = f0.w;
            u[4] = f1.x;  u[5] = f1.y;  u[6] = f1.z;  u[7] = f1.w;
        } else {
            const h8 xv = __builtin_bit_cast(h8, r0), bv = __builtin_bit_cast(h8, r1);
#pragma unroll
            for (int i = 0; i < 8; ++i) u[i] = (float)xv[i] * (float)bv[i];
        }
    }
};

template <bool STAGE_A>
__device__ inline float load_u_scalar(const DbfStage& st, const uint16_t* x, int bi, int l) {
    if (STAGE_A) return st.t[(size_t)bi * st.t_stride + l];
    return half_bits_to_float(x[(size_t)bi * st.cols + l]) * half_bits_to_float(st.in_scale[l]);
}

__device__ inline int quantise(float u, float inv) {
    float f = rintf(u * inv);
    f = fminf(fmaxf(f, -QMAX), QMAX);
    return (int)f;
}

template <bool STAGE_A, int NCG>
__global__ __launch_bounds__(256) void dbf_stage_mfma_kernel(const DbfStage* __restrict__ table,
                                                             const DbfWorkItem* __restrict__ work,
                                                             const uint16_t* __restrict__ x_base,
                                                             uint16_t* __restrict__ y_base,
                                                             int batch, int ch_tiles) {
    extern __shared__ __align__(16) unsigned char smem[];
    int* red = reinterpret_cast<int*>(smem);                                   // [NCG][8][64][4]
    Misc* misc = reinterpret_cast<Misc*>(smem + NCG * 8192);
    signed char* xq = reinterpret_cast<signed char*>(smem + NCG * 8192 + 512);  // [ncols][chs]

    const DbfWorkItem wi = work[blockIdx.x];
    const DbfStage st = table[wi.layer];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int ncols = 2 * batch;
    const int chs = ch_tiles * DBF_TILE_COLS + XQ_PAD;
    const uint16_t* x = x_base + st.x_off * batch;
    uint16_t* y = y_base + st.y_off * batch;

    // sign bits of this workgroup's row tiles: one contiguous span, addressed through a buffer
    // resource so that out-of-range offsets read as zero without touching memory
    const uint8_t* span = st.bits + (size_t)wi.rt0 * st.n_ct * DBF_TILE_BYTES;
    const uint64_t span_addr = reinterpret_cast<uint64_t>(span);
    v4u rsrc;  // raw buffer descriptor: base, stride 0, size in bytes, 32-bit raw data format
    rsrc.x = __builtin_amdgcn_readfirstlane((unsigned)span_addr);
    rsrc.y = __builtin_amdgcn_readfirstlane((unsigned)(span_addr >> 32) & 0xFFFFu);
    rsrc.z = __builtin_amdgcn_readfirstlane((unsigned)(wi.nrt * st.n_ct * DBF_TILE_BYTES));
    rsrc.w = 0x00020000u;
    const unsigned lane_off = lane * 16;

    // Tile cursor of the prefetcher: row tile p_rt (local), step p_i of the chunk.  Step i of a
    // wavefront is column tile c0 + w + 4*i; steps are padded to a multiple of PF per row tile.
    //
    // The loads are issued by inline assembly and waited for by hand (wait_slot): the compiler
    // does not see them, so it cannot serialise the pipeline with a full vmcnt(0) wait at the
    // top of the loop.  Loads complete in issue order; when slot j is consumed exactly PF-1
    // younger tile loads are outstanding, so vmcnt(PF-1) is the exact wait.  Any other memory
    // operation the compiler issues in between only makes that wait more conservative.
    int c0 = 0;
    int cend = min(st.n_ct, ch_tiles);
    int steps = (((cend - c0 + 3) >> 2) + PF - 1) / PF * PF;
    int p_rt = 0, p_i = 0;
    v4u buf[PF];
    auto fetch = [&](v4u& dst) {
        const int ct = c0 + w + 4 * p_i;
        const int ok = (int)(p_rt < wi.nrt) & (int)(ct < cend);
        const unsigned off = (unsigned)(p_rt * st.n_ct + ct) * DBF_TILE_BYTES;
        const unsigned voff = lane_off + (ok ? off : OOB);
#if DBF_ASM_LOADS
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(dst) : "v"(voff), "s"(rsrc) : "memory");
#else
        dst = __builtin_amdgcn_raw_buffer_load_b128(
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(span), 0, (int)rsrc.z, 0x00020000), voff, 0, 0);
#endif
        const int wrap = (int)(p_i + 1 == steps);
        p_i = wrap ? 0 : p_i + 1;
        p_rt += wrap;
    };
    auto wait_slot = [](v4u& slot) {
#if DBF_ASM_LOADS
        asm volatile("s_waitcnt vmcnt(%1)" : "+v"(slot) : "n"(PF - 1) : "memory");
#endif
    };
#pragma unroll
    for (int j = 0; j < PF; ++j) fetch(buf[j]);  // in flight during the prologue

    // ---- prologue: per batch row max|u|, then the fixed-point scale ----------------------
    const int nvec = st.n_ct * 8;  // vector items of 8 values, padding included
    const bool fast = STAGE_A || ((st.cols & 7) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0);
    const int nvec_x = st.cols >> 3;
    for (int bi = 0; bi < batch; ++bi) {
        float mx = 0.f;
        if (fast) {
            for (int base = 0; base < nvec; base += 256 * UNR) {
                InputVec<STAGE_A> iv[UNR];
#pragma unroll
                for (int j = 0; j < UNR; ++j) {
                    const int v = base + 256 * j + tid;
                    if (v < nvec) iv[j].load(st, x, bi, v, v < nvec_x);
                }
#pragma unroll
                for (int j = 0; j < UNR; ++j) {
                    const int v = base + 256 * j + tid;
                    if (v < nvec) {
                        float u[8];
                        iv[j].get(u);
#pragma unroll
                        for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(u[i]));
                    }
                }
            }
        } else {
            for (int l = tid; l < st.cols; l += 256) mx = fmaxf(mx, fabsf(load_u_scalar<STAGE_A>(st, x, bi, l)));
        }
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
    // operand row this lane feeds to the matrix instruction (unused columns alias a valid row)
    int xrow[NCG];
#pragma unroll
    for (int gi = 0; gi < NCG; ++gi) {
        const int col = 16 * gi + c;
        xrow[gi] = (col < ncols ? col : col % ncols) * chs + 16 * g;
    }
    const int xo_max = (ch_tiles - 1) * 64;  // padded steps read a valid (ignored) operand
    // epilogue coordinates: thread -> (row rho of the tile, batch rows bi = tid>>7, +2, ...)
    const int rho = tid & 127;
    const int e_s = rho >> 4, e_g = (rho & 15) >> 2, e_i = rho & 3;

    for (;;) {  // chunks of columns (a single one unless the batch is large)
        // ---- quantise columns [64*c0, 64*cend) of every batch row into LDS ----------------
        for (int bi = 0; bi < batch; ++bi) {
            const float inv = misc->inv[bi];
            int local = 0;
            signed char* hi_row = xq + (2 * bi) * chs;
            signed char* lo_row = xq + (2 * bi + 1) * chs;
            if (fast) {
                const int v0 = c0 * 8, v1 = cend * 8;
                for (int base = v0; base < v1; base += 256 * UNR) {
                    InputVec<STAGE_A> iv[UNR];
#pragma unroll
                    for (int j = 0; j < UNR; ++j) {
                        const int v = base + 256 * j + tid;
                        if (v < v1) iv[j].load(st, x, bi, v, v < nvec_x);
                    }
#pragma unroll
                    for (int j = 0; j < UNR; ++j) {
                        const int v = base + 256 * j + tid;
                        if (v < v1) {
                            float u[8];
                            iv[j].get(u);
                            unsigned hi4[2] = {0, 0}, lo4[2] = {0, 0};
#pragma unroll
                            for (int i = 0; i < 8; ++i) {
                                const int q = quantise(u[i], inv);
                                const int lo = ((q + 128) & 255) - 128;
                                const int hi = (q - lo) >> 8;
                                hi4[i >> 2] |= (unsigned)(hi & 255) << (8 * (i & 3));
                                lo4[i >> 2] |= (unsigned)(lo & 255) << (8 * (i & 3));
                                local += q;
                            }
                            *reinterpret_cast<uint2*>(hi_row + (v - v0) * 8) = make_uint2(hi4[0], hi4[1]);
                            *reinterpret_cast<uint2*>(lo_row + (v - v0) * 8) = make_uint2(lo4[0], lo4[1]);
                        }
                    }
                }
            } else {
                for (int l = c0 * 64 + tid; l < cend * 64; l += 256) {
                    const int q = l < st.cols ? quantise(load_u_scalar<STAGE_A>(st, x, bi, l), inv) : 0;
                    const int lo = ((q + 128) & 255) - 128;
                    const int hi = (q - lo) >> 8;
                    hi_row[l - c0 * 64] = (signed char)hi;
                    lo_row[l - c0 * 64] = (signed char)lo;
                    local += q;
                }
            }
            local = wave_sum(local);
            if (lane == 0) atomicAdd(&misc->sigma[bi], local);
        }
        __syncthreads();
        const bool last_chunk = cend >= st.n_ct;

        for (int rtl = 0; rtl < wi.nrt; ++rtl) {
            if (c0 == 0) {
#pragma unroll
                for (int gi = 0; gi < NCG; ++gi)
#pragma unroll
                    for (int s = 0; s < 8; ++s) acc[gi][s] = (v4i){0, 0, 0, 0};
            }
            // ---- stream this wavefront's tiles of (row tile, chunk) -----------------------
            // Slot j is consumed and then refilled in place, so PF-1 loads stay in flight and
            // no register copies are needed; the operand of the next step is read from LDS
            // one step ahead.
            v4i xop[NCG], xnext[NCG];
#pragma unroll
            for (int gi = 0; gi < NCG; ++gi)
                xnext[gi] = *reinterpret_cast<const v4i*>(xq + xrow[gi] + min(w * 64, xo_max));
            for (int i0 = 0; i0 < steps; i0 += PF) {
#pragma unroll
                for (int j = 0; j < PF; ++j) {
                    const int xo = (w + 4 * (i0 + j + 1)) * 64;  // operand offset of the next step
#pragma unroll
                    for (int gi = 0; gi < NCG; ++gi) {
                        xop[gi] = xnext[gi];
                        xnext[gi] = *reinterpret_cast<const v4i*>(xq + xrow[gi] + min(xo, xo_max));
                    }
                    wait_slot(buf[j]);
#pragma unroll
                    for (int s = 0; s < 8; ++s) {
                        const uint32_t msk = 0x01010101u << s;
                        v4i a;
                        a.x = (int)(buf[j].x & msk);
                        a.y = (int)(buf[j].y & msk);
                        a.z = (int)(buf[j].z & msk);
                        a.w = (int)(buf[j].w & msk);
#pragma unroll
                        for (int gi = 0; gi < NCG; ++gi)
                            acc[gi][s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, xop[gi], acc[gi][s], 0, 0, 0);
                    }
                    fetch(buf[j]);
                }
            }
            if (!last_chunk) continue;  // (only with nrt == 1) keep accumulating over chunks

            // ---- combine the four wavefronts (integer adds: exact, order independent) -----
#pragma unroll
            for (int gi = 0; gi < NCG; ++gi) {
                if (16 * gi + c < ncols) {
#pragma unroll
                    for (int s = 0; s < 8; ++s)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            atomicAdd(&red[((gi * 8 + s) * 64 + lane) * 4 + i], acc[gi][s][i]);
                }
            }
            __syncthreads();
            // result element (row 4*g'+i of group s, column) sits in lane 16*g'+column
            const int row = (wi.rt0 + rtl) * DBF_TILE_ROWS + rho;
            const float rscale = half_bits_to_float(st.row_scale[row]);
            for (int bi = tid >> 7; bi < batch; bi += 2) {
                const int col = 2 * bi;
                const int gi = col >> 4, cc = col & 15;
                int* ph = &red[((gi * 8 + e_s) * 64 + 16 * e_g + cc) * 4 + e_i];
                int vh = ph[0], vl = ph[4];
                ph[0] = 0;  // ready for the next row tile
                ph[4] = 0;
                if (e_s < 7) {
                    vh >>= e_s;
                    vl >>= e_s;
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
            __syncthreads();
        }
        if (last_chunk) break;
        // next chunk (reached only with nrt == 1): restart the tile cursor there
        __syncthreads();  // every wavefront is done reading this chunk's operand
        c0 = cend;
        cend = min(st.n_ct, c0 + ch_tiles);
        steps = (((cend - c0 + 3) >> 2) + PF - 1) / PF * PF;
        p_rt = 0;
        p_i = 0;
#pragma unroll
        for (int j = 0; j < PF; ++j) fetch(buf[j]);
    }
}

}  // namespace

int dbf_mfma_chunk_tiles(int batch, int max_cols) {
    const int ncg = batch > 8 ? 2 : 1;
    const int ncols = 2 * batch;
    const int budget = ncg == 2 ? 40960 : 32768;  // LDS bytes for the quantised operand
    int ch_tiles = ((budget / ncols - XQ_PAD) / DBF_TILE_COLS) & ~3;
    const int need = (dbf_col_tiles(max_cols) + 3) & ~3;
    if (ch_tiles > need) ch_tiles = need;
    if (ch_tiles < 4) ch_tiles = 4;
    return ch_tiles;
}

hipError_t dbf_launch_stage_mfma(bool stage_a, const DbfStage* table, const DbfWorkItem* work,
                                 int blocks, const void* x_base, void* y_base, int batch,
                                 int max_cols, hipStream_t stream) {
    if (blocks <= 0) return hipSuccess;
    const uint16_t* x = static_cast<const uint16_t*>(x_base);
    uint16_t* y = static_cast<uint16_t*>(y_base);
    const int ncg = batch > 8 ? 2 : 1;
    const int ncols = 2 * batch;
    const int ch_tiles = dbf_mfma_chunk_tiles(batch, max_cols);
    const size_t smem = (size_t)ncg * 8192 + 512 + (size_t)ncols * (ch_tiles * DBF_TILE_COLS + XQ_PAD);
    if (ncg == 1) {
        if (stage_a)
            hipLaunchKernelGGL((dbf_stage_mfma_kernel<true, 1>), dim3(blocks), dim3(256), smem, stream,
                               table, work, x, y, batch, ch_tiles);
        else
            hipLaunchKernelGGL((dbf_stage_mfma_kernel<false, 1>), dim3(blocks), dim3(256), smem, stream,
                               table, work, x, y, batch, ch_tiles);
    } else {
        if (stage_a)
            hipLaunchKernelGGL((dbf_stage_mfma_kernel<true, 2>), dim3(blocks), dim3(256), smem, stream,
                               table, work, x, y, batch, ch_tiles);
        else
            hipLaunchKernelGGL((dbf_stage_mfma_kernel<false, 2>), dim3(blocks), dim3(256), smem, stream,
                               table, work, x, y, batch, ch_tiles);
    }
    return hipGetLastError();
}
