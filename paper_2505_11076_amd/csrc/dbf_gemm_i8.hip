// Prefill with the int8 matrix cores as the adder: the decode trick (dbf_gemv_mfma.hip) for T tokens.
//
//   quantise:  u = X . b per token, rounded once to 16-bit fixed point, split into two int8 planes
//   stage 1:   mid = ((X . b) B^T) . m      (T x k, fp32)   contraction over n_in
//   quantise:  mid per token -> two int8 planes
//   stage 2:   Y   = (mid A^T) . a          (T x n_out, fp16) contraction over k
//
// (forward-pass expression of the paper, section 3; the paper times batch 1 only, so this design
// is not taken from it).  Compared with the fp16 path (dbf_gemm_mfma.hip):
//   * the A operand of v_mfma_i32_16x16x64_i8 is the masked sign bytes, one AND per register
//     (0.25 vector-ALU operations per sign instead of 1), and one instruction covers 64 columns;
//   * the sums are exact integers: acc_s = 2^s * sum over set bits of q, so
//     sum(+-q) = 2 (acc_s >> s) - sum(q); the only roundings left are the two 16-bit
//     quantisations (relative 2^-16 of the row maximum) and the fp16 output;
//   * hi and lo planes are separate instructions with separate accumulators: twice the
//     instructions at twice the int8 rate.
//
// Work split of a stage: workgroup = 256 rows x 64 tokens, 4 wavefronts; wavefront w owns row tile
// (w & 1) and the token half (w >> 1): 128 rows x 32 tokens = 8 planes x 2 token blocks x
// {hi, lo} = 32 accumulator tiles (128 registers).  Twice as many workgroups as compute units at
// 4096 rows x 2048 tokens, i.e. two wavefronts per SIMD.  The 64-token slice of the quantised
// operand (2 planes x 64 tokens x 64 bytes per step) is staged in LDS, double buffered; sign
// tiles and operand columns of step kt + 4 are requested while step kt is computed, by loads
// issued and waited for by hand (see the stage kernel).
#include "dbf_kernels.h"
#include "dbf_wave.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));

constexpr float QMAX = 32512.f;     // 127*256: largest |q| so that hi and lo fit int8
constexpr int QI_TOKENS = 64;       // tokens per workgroup
constexpr int QI_ROWTILES = 2;      // 128-row tiles per workgroup
constexpr int QI_TROW = 64 + 16;    // LDS bytes per (plane, token): 64 operand bytes + bank padding
constexpr int QI_PLANE = QI_TOKENS * QI_TROW;
constexpr int QI_DEPTH = 4;         // steps requested ahead
constexpr int QI_TB = 2;            // 16-token blocks per wavefront: 8 planes x 2 x {hi, lo} = 128 accumulator registers
constexpr int QI_TSPLIT = QI_TOKENS / (16 * QI_TB);       // token slices of a row tile
// 1: workgroups that read the same operand slice are renumbered onto one compute die (one L2); 0: launch order
#ifndef DBF_QI_XCD_REMAP
#define DBF_QI_XCD_REMAP 1
#endif

constexpr int QI_WAVES = QI_ROWTILES * QI_TSPLIT;
constexpr int QI_OCC = 2;           // wavefronts per SIMD (the accumulators leave room for no more)
constexpr int QI_THREADS = 64 * QI_WAVES;
constexpr int SPLIT_CNT_STRIDE = 32;  // unsigned ints between the arrival counters of two column-split groups: 128 bytes
constexpr int QI_STAGE_BYTES = 2 * QI_TOKENS * 64 / QI_THREADS;  // operand bytes a thread stages per step
static_assert(QI_STAGE_BYTES == 32, "staging is two 16-byte pieces per thread");


// ---------------------------------------------------------------------------------------------
// Quantisation of token rows: q = rint(u * 32512 / max|u|), hi/lo int8 planes.
//   FROM_F32 = false: u = x (fp16) * col_scale (fp16, zero padded)      (input of stage 1)
//   FROM_F32 = true:  u = src (fp32, leading dimension ld)               (input of stage 2)
// Output layout ("step major"): byte ((kt * Tp + token) * 2 + plane) * 64 + j holds plane (0 = hi,
// 1 = lo) of column 64 kt + j of `token`; Tp = T rounded up to 64.  The 64 tokens x 2 planes x 64
// bytes a workgroup of the stage kernel stages per step are then 8 KiB of contiguous memory.
// Zeros beyond `cols`; scale[token] = max|u| / 32512, sigma[token] = sum of q.
// ---------------------------------------------------------------------------------------------
struct QuantArgs {
    const void* src;
    const uint16_t* col_scale;
    signed char* dst;
    float* scale;
    int* sigma;
    int T, Tp, cols, kp;
    long long ld;     // elements between token rows of src
    int vec_ok;       // rows can be read in 16-byte (fp16) / 32-byte (fp32) pieces
    v4u* zero;        // 16-byte pieces this launch clears on the side (the column splits' sums and counters), or NULL
    unsigned zero_v4;
};

// The integer sums and arrival counters of the stage kernels' column splits must start at zero, and a caller's
// workspace holds anything: the first quantiser launch of a call, which runs before either stage, clears them,
// its threads sharing the pieces evenly.
__device__ inline void zero_share(const QuantArgs& a) {
    if (!a.zero) return;
    const unsigned n_thr = gridDim.x * blockDim.x;
    for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < a.zero_v4; i += n_thr) a.zero[i] = (v4u){0, 0, 0, 0};
}

template <bool FROM_F32>
__device__ inline void load8(const QuantArgs& a, int token, int v, float (&u)[8]) {
    // columns 8v .. 8v+7 (v < kp/8); zero beyond `cols`
    const int c0 = 8 * v;
    if (FROM_F32) {
        const float* row = static_cast<const float*>(a.src) + (size_t)token * a.ld;
        if (a.vec_ok && c0 + 8 <= a.cols) {
            const v4f f0 = *reinterpret_cast<const v4f*>(row + c0), f1 = *reinterpret_cast<const v4f*>(row + c0 + 4);
            u[0] = f0.x;  u[1] = f0.y;  u[2] = f0.z;  u[3] = f0.w;
            u[4] = f1.x;  u[5] = f1.y;  u[6] = f1.z;  u[7] = f1.w;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i) u[i] = c0 + i < a.cols ? row[c0 + i] : 0.f;
        }
    } else {
        const uint16_t* row = static_cast<const uint16_t*>(a.src) + (size_t)token * a.ld;
        if (a.vec_ok && c0 + 8 <= a.cols) {
            const h8 xv = *reinterpret_cast<const h8*>(row + c0);
            const h8 bv = *reinterpret_cast<const h8*>(a.col_scale + c0);
            u[0] = (float)xv.s0 * (float)bv.s0;  u[1] = (float)xv.s1 * (float)bv.s1;
            u[2] = (float)xv.s2 * (float)bv.s2;  u[3] = (float)xv.s3 * (float)bv.s3;
            u[4] = (float)xv.s4 * (float)bv.s4;  u[5] = (float)xv.s5 * (float)bv.s5;
            u[6] = (float)xv.s6 * (float)bv.s6;  u[7] = (float)xv.s7 * (float)bv.s7;
        } else {
#pragma unroll
            for (int i = 0; i < 8; ++i)
                u[i] = c0 + i < a.cols ? (float)__builtin_bit_cast(_Float16, row[c0 + i]) *
                                             (float)__builtin_bit_cast(_Float16, a.col_scale[c0 + i])
                                       : 0.f;
        }
    }
}

// Quantises eight values and stores their two planes; returns the sum of the q.
__device__ inline int quantise_store(const QuantArgs& a, int token, int v, const float (&u)[8], float inv) {
    unsigned hi4[2] = {0, 0}, lo4[2] = {0, 0};
    int sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        float f = rintf(u[i] * inv);
        f = fminf(fmaxf(f, -QMAX), QMAX);
        const int q = (int)f;
        const int lo = ((q + 128) & 255) - 128;
        const int hi = (q - lo) >> 8;
        hi4[i >> 2] |= (unsigned)(hi & 255) << (8 * (i & 3));
        lo4[i >> 2] |= (unsigned)(lo & 255) << (8 * (i & 3));
        sum += q;
    }
    signed char* d = a.dst + (((size_t)(v >> 3) * a.Tp + token) * 2) * 64 + 8 * (v & 7);
    *reinterpret_cast<uint2*>(d) = make_uint2(hi4[0], hi4[1]);
    *reinterpret_cast<uint2*>(d + 64) = make_uint2(lo4[0], lo4[1]);
    return sum;
}

// One wavefront per token (four tokens per workgroup, no LDS, no barriers).  Rows of up to 4096
// columns are held in registers between the max pass and the quantisation; longer rows are read
// twice (the second read hits in L2).
template <bool FROM_F32>
__global__ __launch_bounds__(256) void dbf_quantise_rows_kernel(const QuantArgs a) {
    zero_share(a);
    constexpr int HOLD = 8;  // vectors of 8 columns a lane can hold
    const int lane = threadIdx.x & 63;
    const int token = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (token >= a.T) return;
    const int nvec = a.kp >> 3;
    float mx = 0.f;
    int local = 0;
    if (nvec <= 64 * HOLD) {
        float u[HOLD][8];
#pragma unroll
        for (int r = 0; r < HOLD; ++r) {
            const int v = lane + 64 * r;
            if (v < nvec) {
                load8<FROM_F32>(a, token, v, u[r]);
#pragma unroll
                for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(u[r][i]));
            }
        }
        mx = dbf_wave_max(mx);
        const float inv = mx > 0.f ? QMAX / mx : 0.f;
#pragma unroll
        for (int r = 0; r < HOLD; ++r) {
            const int v = lane + 64 * r;
            if (v < nvec) local += quantise_store(a, token, v, u[r], inv);
        }
    } else {
        for (int v = lane; v < nvec; v += 64) {
            float u[8];
            load8<FROM_F32>(a, token, v, u);
#pragma unroll
            for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(u[i]));
        }
        mx = dbf_wave_max(mx);
        const float inv = mx > 0.f ? QMAX / mx : 0.f;
        for (int v = lane; v < nvec; v += 64) {
            float u[8];
            load8<FROM_F32>(a, token, v, u);
            local += quantise_store(a, token, v, u, inv);
        }
    }
    local = dbf_wave_sum(local);
    if (lane == 0) {
        a.scale[token] = mx / QMAX;
        a.sigma[token] = local;
    }
}

// One workgroup per token, the row held in registers (HOLD vector items of 8 columns per thread: rows of up to
// 2048 * HOLD columns that can be read in 16-byte pieces).  Straight-line: every load of the row is issued before
// anything waits (vector items beyond the row are read as its last one and zeroed afterwards); the four
// wavefronts exchange their maxima and sums through LDS.  With 8192 wavefronts of little work each instead of
// 2048 of much, the launch is as long as one memory round trip and a little arithmetic.
template <bool FROM_F32, int HOLD>
__global__ __launch_bounds__(256) void dbf_quantise_rows_held_kernel(const QuantArgs a) {
    zero_share(a);
    __shared__ float wmax[4];
    __shared__ int wsum[4];
    const int token = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nvec = a.kp >> 3, nreal = a.cols >> 3;
    float u[HOLD][8];
    if (FROM_F32) {
        const float* row = static_cast<const float*>(a.src) + (size_t)token * a.ld;
        v4f f0[HOLD], f1[HOLD];
#pragma unroll
        for (int r = 0; r < HOLD; ++r) {
            const int c0 = 8 * min(tid + 256 * r, nreal - 1);
            f0[r] = *reinterpret_cast<const v4f*>(row + c0);
            f1[r] = *reinterpret_cast<const v4f*>(row + c0 + 4);
        }
#pragma unroll
        for (int r = 0; r < HOLD; ++r) {
            const bool in = tid + 256 * r < nreal;
            u[r][0] = in ? f0[r].x : 0.f;  u[r][1] = in ? f0[r].y : 0.f;
            u[r][2] = in ? f0[r].z : 0.f;  u[r][3] = in ? f0[r].w : 0.f;
            u[r][4] = in ? f1[r].x : 0.f;  u[r][5] = in ? f1[r].y : 0.f;
            u[r][6] = in ? f1[r].z : 0.f;  u[r][7] = in ? f1[r].w : 0.f;
        }
    } else {
        const uint16_t* row = static_cast<const uint16_t*>(a.src) + (size_t)token * a.ld;
        h8 xv[HOLD], bv[HOLD];
#pragma unroll
        for (int r = 0; r < HOLD; ++r) {
            const int c0 = 8 * min(tid + 256 * r, nreal - 1);
            xv[r] = *reinterpret_cast<const h8*>(row + c0);
            bv[r] = *reinterpret_cast<const h8*>(a.col_scale + c0);
        }
#pragma unroll
        for (int r = 0; r < HOLD; ++r) {
            const bool in = tid + 256 * r < nreal;
#pragma unroll
            for (int i = 0; i < 8; ++i) u[r][i] = in ? (float)xv[r][i] * (float)bv[r][i] : 0.f;
        }
    }
    float mx = 0.f;
#pragma unroll
    for (int r = 0; r < HOLD; ++r)
#pragma unroll
        for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(u[r][i]));
    mx = dbf_wave_max(mx);
    if (lane == 0) wmax[w] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    const float inv = mx > 0.f ? QMAX / mx : 0.f;
    int local = 0;
#pragma unroll
    for (int r = 0; r < HOLD; ++r) {
        const int v = tid + 256 * r;
        if (v < nvec) local += quantise_store(a, token, v, u[r], inv);
    }
    local = dbf_wave_sum(local);
    if (lane == 0) wsum[w] = local;
    __syncthreads();
    if (tid == 0) {
        a.scale[token] = mx / QMAX;
        a.sigma[token] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    }
}

// One workgroup per token: for rows too long to hold in a wavefront's registers.
template <bool FROM_F32>
__global__ __launch_bounds__(256) void dbf_quantise_rows_block_kernel(const QuantArgs a) {
    zero_share(a);
    __shared__ float wmax[4];
    __shared__ int wsum[4];
    const int token = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int nvec = a.kp >> 3;
    float mx = 0.f;
    for (int v = tid; v < nvec; v += 256) {
        float u[8];
        load8<FROM_F32>(a, token, v, u);
#pragma unroll
        for (int i = 0; i < 8; ++i) mx = fmaxf(mx, fabsf(u[i]));
    }
    mx = dbf_wave_max(mx);
    if (lane == 0) wmax[w] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(wmax[0], wmax[1]), fmaxf(wmax[2], wmax[3]));
    const float inv = mx > 0.f ? QMAX / mx : 0.f;
    int local = 0;
    for (int v = tid; v < nvec; v += 256) {
        float u[8];
        load8<FROM_F32>(a, token, v, u);   // second read of the row: L2 resident
        unsigned hi4[2] = {0, 0}, lo4[2] = {0, 0};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float f = rintf(u[i] * inv);
            f = fminf(fmaxf(f, -QMAX), QMAX);
            const int q = (int)f;
            const int lo = ((q + 128) & 255) - 128;
            const int hi = (q - lo) >> 8;
            hi4[i >> 2] |= (unsigned)(hi & 255) << (8 * (i & 3));
            lo4[i >> 2] |= (unsigned)(lo & 255) << (8 * (i & 3));
            local += q;
        }
        signed char* d = a.dst + (((size_t)(v >> 3) * a.Tp + token) * 2) * 64 + 8 * (v & 7);
        *reinterpret_cast<uint2*>(d) = make_uint2(hi4[0], hi4[1]);
        *reinterpret_cast<uint2*>(d + 64) = make_uint2(lo4[0], lo4[1]);
    }
    local = dbf_wave_sum(local);
    if (lane == 0) wsum[w] = local;
    __syncthreads();
    if (tid == 0) {
        a.scale[token] = mx / QMAX;
        a.sigma[token] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
    }
}

// ---------------------------------------------------------------------------------------------
// One stage: out[token][row] = rscale[row] * scale[token] * sum_col sign(row, col) * q[token][col]
// ---------------------------------------------------------------------------------------------
struct StageArgs {
    const uint8_t* bits;        // tiled sign matrix: n_rt x n_ct tiles
    const uint16_t* row_scale;  // fp16 [n_rt*128] (m or a, zero padded)
    const signed char* xq;      // [n_ct][Tp][2][64] quantised operand (step major, see above)
    const float* scale;         // [T]
    const int* sigma;           // [T]
    void* out;                  // OUT_F32: float [T][ldo]; else fp16 [T][ldo]
    int n_rt, n_ct, T, Tp, ldo;
    int n_valid;                // output rows to store
    // column splits (SPLIT kernels only): grid.z workgroups share the column steps of a (row group, token block);
    // each adds its exact integer sums into slab, the last one to arrive (cnt) scales and stores them and leaves
    // both at zero
    int splits;
    int* slab;                  // int32 [token blocks][row groups][QI_WAVES][QI_TB * 8 * 4][64 lanes], zero on entry
    unsigned* cnt;              // [token blocks][row groups], zero on entry
};

// SPLIT: few tokens leave most of the chip idle (a workgroup per 256 rows x 64 tokens walks all column steps:
// 16 workgroups for 64 tokens of a 4096-row stage), so grid.z workgroups take a share of the column steps each.
// Their sums are exact integers, so adding them in any order gives the bits of the unsplit kernel.
template <bool OUT_F32, bool SPLIT>
__global__ __launch_bounds__(QI_THREADS) __attribute__((amdgpu_waves_per_eu(QI_OCC, QI_OCC)))
void dbf_gemm_i8_stage_kernel(const StageArgs a) {
    __shared__ __align__(16) unsigned char xs[2][2 * QI_PLANE];
    __shared__ int last_split;

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    // Workgroups are handed to the 8 compute dies in turn (linear id modulo 8) and each die has its own L2.
    // All workgroups of a token block read the same operand slice, so they are renumbered to share a die:
    // die d takes a contiguous range of the (token block, row group) pairs, row group fastest.
#if DBF_QI_XCD_REMAP
    const unsigned n_wg = gridDim.x * gridDim.y, lin = blockIdx.x + gridDim.x * blockIdx.y;
    const unsigned die = lin & 7, slot = lin >> 3, per = n_wg >> 3, extra = n_wg & 7;
    const unsigned vid = die * per + (die < extra ? die : extra) + slot;
    const int bx = (int)(vid % gridDim.x), by = (int)(vid / gridDim.x);
#else
    const int bx = blockIdx.x, by = blockIdx.y;
#endif
    const int token0 = by * QI_TOKENS;
    const int th = w / QI_ROWTILES;                          // token slice of this wavefront
    int rt = bx * QI_ROWTILES + (w % QI_ROWTILES);           // its row tile
    const bool active = rt < a.n_rt;                         // beyond the matrix: compute on tile 0, store nothing
    if (!active) rt = 0;

    // staging role: thread -> (token, plane, 32-byte half of the 64 operand bytes of a step)
    // (the 8 KiB of a step are contiguous in memory: thread t takes bytes [SB*t, SB*t + SB))
    constexpr int SB = QI_STAGE_BYTES;
    const int s_tok = (tid * SB) >> 7, s_plane = ((tid * SB) >> 6) & 1, s_half = (tid * SB) & 63;
    // (tokens in [T, Tp) hold whatever the workspace held: they are computed and never stored)
    const size_t s_step = (size_t)a.Tp * 128;                // bytes between steps
    unsigned char* s_dst0 = xs[0] + s_plane * QI_PLANE + s_tok * QI_TROW + s_half;
    unsigned char* s_dst1 = xs[1] + s_plane * QI_PLANE + s_tok * QI_TROW + s_half;

    v4i acc[8][QI_TB][2];  // [plane s][token block][hi, lo]
#pragma unroll
    for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int tb = 0; tb < QI_TB; ++tb) {
            acc[s][tb][0] = (v4i){0, 0, 0, 0};
            acc[s][tb][1] = (v4i){0, 0, 0, 0};
        }

    // Software pipeline with hand-issued loads.  The sign tile and the operand bytes of step kt + QI_DEPTH are
    // requested at the end of step kt by inline assembly and waited for by hand: the compiler does not see
    // these loads, so it cannot drain the whole pipeline with a vmcnt(0) wait at the loop's back edge (which
    // it does for loads it tracks: once per QI_DEPTH steps every wavefront then sits out a full memory
    // latency).  Loads complete in issue order.  A step's group is issued as (x0, x1, bq); at the top of step
    // kt the groups of steps kt+1 .. kt+3 are in flight behind bq of step kt, and the step needs bq(kt),
    // x0(kt+1), x1(kt+1): bq(kt+1) and the two younger groups may stay outstanding = 1 + 3 + 3 loads.
    static_assert(QI_DEPTH == 4 && QI_STAGE_BYTES == 32, "the wait counts below are written for this pipeline");
    v4u bq[QI_DEPTH], x0[QI_DEPTH], x1[QI_DEPTH];
    const int last_ct = a.n_ct - 1;
    // this workgroup's column steps: all of them, or the blockIdx.z-th share
    const int kt_lo = SPLIT ? (int)((long long)a.n_ct * blockIdx.z / a.splits) : 0;
    const int kt_hi = SPLIT ? (int)((long long)a.n_ct * (blockIdx.z + 1) / a.splits) : a.n_ct;
    const unsigned x_voff = (unsigned)(SB * tid), t_voff = (unsigned)(lane * 16);
    const signed char* x_base = a.xq + (size_t)token0 * 128;
    const uint8_t* t_base = a.bits + (size_t)rt * a.n_ct * DBF_TILE_BYTES;
    auto request = [&](int j, int kt) {  // kt is the same for all lanes: the step's part of the address is scalar
        const signed char* xs_ = x_base + (size_t)kt * s_step;
        const uint8_t* ts_ = t_base + (size_t)kt * DBF_TILE_BYTES;
        asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(x0[j]) : "v"(x_voff), "s"(xs_) : "memory");
        asm volatile("global_load_dwordx4 %0, %1, %2 offset:16" : "=v"(x1[j]) : "v"(x_voff), "s"(xs_) : "memory");
        asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(bq[j]) : "v"(t_voff), "s"(ts_) : "memory");
    };
#pragma unroll
    for (int j = 0; j < QI_DEPTH; ++j) request(j, min(kt_lo + j, last_ct));
    asm volatile("s_waitcnt vmcnt(10)" : "+v"(x0[0]), "+v"(x1[0]) : : "memory");
    *reinterpret_cast<v4u*>(s_dst0) = x0[0];
    *reinterpret_cast<v4u*>(s_dst0 + 16) = x1[0];
    __syncthreads();

    const unsigned char* xlane = xs[0] + (16 * QI_TB * th + c) * QI_TROW + 16 * g;

    for (int kt0 = kt_lo; kt0 < kt_hi; kt0 += QI_DEPTH) {
#pragma unroll
        for (int j = 0; j < QI_DEPTH; ++j) {
            const int kt = kt0 + j;
            const int jn = (j + 1) % QI_DEPTH;
            asm volatile("s_waitcnt vmcnt(7)" : "+v"(x0[jn]), "+v"(x1[jn]), "+v"(bq[j]) : : "memory");
            // stage step kt + 1 into the other buffer
            {
                unsigned char* d = (j & 1) ? s_dst0 : s_dst1;
                *reinterpret_cast<v4u*>(d) = x0[jn];
                *reinterpret_cast<v4u*>(d + 16) = x1[jn];
            }
            // A step beyond the matrix contributes nothing if its sign operand is zero (no branch around
            // the matrix instructions); `live` is the same for all lanes and is folded into the plane masks.
            const unsigned live = kt < kt_hi ? 0xFFFFFFFFu : 0u;
            const unsigned char* xb = xlane + (j & 1) * (2 * QI_PLANE);
            v4i xop[QI_TB][2];
#pragma unroll
            for (int tb = 0; tb < QI_TB; ++tb) {
                xop[tb][0] = *reinterpret_cast<const v4i*>(xb + tb * 16 * QI_TROW);
                xop[tb][1] = *reinterpret_cast<const v4i*>(xb + tb * 16 * QI_TROW + QI_PLANE);
            }
            v4i av[8];
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const unsigned msk = (0x01010101u << s) & live;
                av[s].x = (int)(bq[j].x & msk);
                av[s].y = (int)(bq[j].y & msk);
                av[s].z = (int)(bq[j].z & msk);
                av[s].w = (int)(bq[j].w & msk);
                if (s == 7) {
                    // every register of slot j has been read: request step kt + QI_DEPTH into it
                    asm volatile("" : "+v"(av[s]), "+v"(bq[j]), "+v"(x0[j]), "+v"(x1[j]));
                    request(j, min(kt + QI_DEPTH, last_ct));
                }
#pragma unroll
                for (int tb = 0; tb < QI_TB; ++tb) {
                    acc[s][tb][0] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s], xop[tb][0], acc[s][tb][0], 0, 0, 0);
                    acc[s][tb][1] = __builtin_amdgcn_mfma_i32_16x16x64_i8(av[s], xop[tb][1], acc[s][tb][1], 0, 0, 0);
                }
            }
            __syncthreads();
        }
    }
    // the requests of the last QI_DEPTH steps are still in flight: let them land before their registers are reused
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int j = 0; j < QI_DEPTH; ++j) asm volatile("" : "+v"(bq[j]), "+v"(x0[j]), "+v"(x1[j]));

    // ---- epilogue: acc[s][tb][p][i] of lane (g, c) is row 16*s + 4*g + i, token 32*th + 16*tb + c ----
    // (vh * 256 + vl below: the sum of q over the set bits of the row, exact)
    int* const my_sums = SPLIT ? a.slab + (((size_t)by * gridDim.x + bx) * QI_WAVES + w) * (QI_TB * 8 * 4 * 64) + lane : nullptr;
    if (SPLIT) {
        // add this share's sums (lane-major: a wavefront's adds of one value are 64 consecutive words), count the
        // workgroup in, and go on only if it is the last of its (row group, token block)
#pragma unroll
        for (int tb = 0; tb < QI_TB; ++tb) {
            const int token = token0 + 16 * QI_TB * th + 16 * tb + c;
            if (!active || token >= a.T) continue;
#pragma unroll
            for (int s = 0; s < 8; ++s)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    int vh = acc[s][tb][0][i] >> s, vl = acc[s][tb][1][i] >> s;
                    if (s == 7) {
                        vh = -vh;
                        vl = -vl;
                    }
                    __hip_atomic_fetch_add(my_sums + ((tb * 8 + s) * 4 + i) * 64, vh * 256 + vl, __ATOMIC_RELAXED,
                                           __HIP_MEMORY_SCOPE_AGENT);
                }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wavefront's adds have been performed ...
        __syncthreads();                                  // ... and so have the workgroup's
        if (tid == 0) {
            unsigned* cnt = a.cnt + ((size_t)by * gridDim.x + bx) * SPLIT_CNT_STRIDE;  // (a cache line per counter)
            const unsigned before = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            last_split = before == (unsigned)a.splits - 1u;
            if (last_split) __hip_atomic_store(cnt, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (!last_split) return;
    }
    if (!active) return;
#pragma unroll
    for (int tb = 0; tb < QI_TB; ++tb) {
        const int token = token0 + 16 * QI_TB * th + 16 * tb + c;
        if (token >= a.T) continue;
        const float tscale = a.scale[token];
        const int tsigma = a.sigma[token];
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int n0 = rt * DBF_TILE_ROWS + 16 * s + 4 * g;
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int vh = acc[s][tb][0][i] >> s, vl = acc[s][tb][1][i] >> s;
                if (s == 7) {  // the mask 0x80 is -128 as an int8
                    vh = -vh;
                    vl = -vl;
                }
                // (the last share reads the sums of all shares and leaves zeros for the next call)
                const int set_sum = SPLIT ? __hip_atomic_exchange(my_sums + ((tb * 8 + s) * 4 + i) * 64, 0, __ATOMIC_RELAXED,
                                                                  __HIP_MEMORY_SCOPE_AGENT)
                                          : vh * 256 + vl;
                // (2 * the sum of the set bits' q may pass 2^31 on the way to a total that fits: modular arithmetic)
                const int total = (int)(2u * (unsigned)set_sum - (unsigned)tsigma);
                const float rs = (float)__builtin_bit_cast(_Float16, a.row_scale[n0 + i]);
                v[i] = (float)total * tscale * rs;
            }
            if (OUT_F32) {
                float* dst = static_cast<float*>(a.out) + (size_t)token * a.ldo + n0;
                if (n0 + 4 <= a.n_valid) {
                    *reinterpret_cast<v4f*>(dst) = (v4f){v[0], v[1], v[2], v[3]};
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (n0 + i < a.n_valid) dst[i] = v[i];
                }
            } else {
                uint16_t* dst = static_cast<uint16_t*>(a.out) + (size_t)token * a.ldo + n0;
                const bool vec_ok = (a.ldo & 3) == 0 && (reinterpret_cast<uintptr_t>(a.out) & 7) == 0;
                if (vec_ok && n0 + 4 <= a.n_valid) {
                    typedef _Float16 h4 __attribute__((ext_vector_type(4)));
                    *reinterpret_cast<h4*>(dst) = (h4){(_Float16)v[0], (_Float16)v[1], (_Float16)v[2], (_Float16)v[3]};
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (n0 + i < a.n_valid) dst[i] = __builtin_bit_cast(uint16_t, (_Float16)v[i]);
                }
            }
        }
    }
}

// The quantiser for a row length: rows held in registers where they can be read in 16-byte pieces (up to 4096 and up
// to 12288 padded columns), else a wavefront or a workgroup per token that reads value by value / twice.
template <bool FROM_F32>
void launch_quantise(const QuantArgs& q, size_t kp, int T, hipStream_t stream) {
    const bool straight = q.vec_ok && (q.cols & 7) == 0 && q.cols >= 8;
    if (straight && kp <= 4096)
        hipLaunchKernelGGL((dbf_quantise_rows_held_kernel<FROM_F32, 2>), dim3(T), dim3(256), 0, stream, q);
    else if (straight && kp <= 12288)
        hipLaunchKernelGGL((dbf_quantise_rows_held_kernel<FROM_F32, 6>), dim3(T), dim3(256), 0, stream, q);
    else if (kp <= 4096)
        hipLaunchKernelGGL(dbf_quantise_rows_kernel<FROM_F32>, dim3((T + 3) / 4), dim3(256), 0, stream, q);
    else
        hipLaunchKernelGGL(dbf_quantise_rows_block_kernel<FROM_F32>, dim3(T), dim3(256), 0, stream, q);
}

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

// Column splits: in calls of up to SPLIT_MAX_T tokens a stage that would start at most SPLIT_UP_TO_WGS workgroups cuts
// its column steps into SPLIT_SHARES shares (of at least SPLIT_MIN_STEPS steps).  What a share saves is column steps
// (0.6 us each); what it costs is an atomic add per output and share, so it pays only while the stage has few
// outputs.  Measured, microseconds per call without / with 4 shares (2 and 8 in brackets where they differ much):
//   4096 x 4096, k = 4096      33 tokens 65.8 / 46.5   64: 67.2 / 50.6   128: 68.1 / 57.3 (8: 67.6)   256: 69.8 / 67.0
//                              512: 72.0 / 92.9 (2: 81.1)
//   11008 -> 4096, k = 5970    33: 121.5 / 64.1 (8: 61.0)   64: 123.0 / 69.0   128: 123.5 / 75.3   256: 124.3 / 92.5
//                              512: 129.4 / 136.2
//   4096 -> 11008, k = 2985    33: 60.6 / 48.2   64: 61.7 / 53.3   128: 62.6 / 63.5   256: 65.2 / 86.7
constexpr int SPLIT_MAX_T = 512;
constexpr int SPLIT_UP_TO_WGS = 64;
constexpr int SPLIT_SHARES = 4;
constexpr int SPLIT_MIN_STEPS = 8;

int pick_splits(int row_groups, unsigned tok_blocks, int n_ct) {
    const int forced = dbf_tune(DBF_TUNE_GEMM_SPLITS);
    int s = 1;
    if (forced > 0) {
        s = forced;
    } else {
        // (a long column walk -- 128 steps and more, i.e. 8192 columns -- still pays at twice as many workgroups:
        //  11008 -> 4096, k = 5970 at 256 tokens 114 -> 93 us)
        const long long wgs = (long long)row_groups * tok_blocks;
        if (wgs > SPLIT_UP_TO_WGS && !(wgs <= 2 * SPLIT_UP_TO_WGS && n_ct >= 128)) return 1;
        s = SPLIT_SHARES;
        if (s > n_ct / SPLIT_MIN_STEPS) s = n_ct / SPLIT_MIN_STEPS;
    }
    if (s > n_ct) s = n_ct;
    if (s > 65535) s = 65535;
    return s < 1 ? 1 : s;
}

// workspace carve-up (all sections 256-byte aligned)
struct I8Workspace {
    size_t xq1, sc1, sg1, mid, xq2, sc2, sg2, slab, cnt, total, total_without_splits;
};
inline I8Workspace i8_workspace(const dbf_layer* L, int T) {
    const size_t kp1 = (size_t)dbf_col_tiles(L->n_in) * DBF_TILE_COLS;
    const size_t kp2 = (size_t)dbf_col_tiles(L->k) * DBF_TILE_COLS;
    const size_t ks = (size_t)dbf_row_tiles(L->k) * DBF_TILE_ROWS;
    const size_t Tp = ((size_t)T + 63) & ~(size_t)63;
    I8Workspace w;
    size_t off = 0;
    w.xq1 = off;  off = align256(off + Tp * 2 * kp1);
    w.sc1 = off;  off = align256(off + (size_t)T * 4);
    w.sg1 = off;  off = align256(off + (size_t)T * 4);
    w.mid = off;  off = align256(off + (size_t)T * ks * 4);
    w.xq2 = off;  off = align256(off + Tp * 2 * kp2);
    w.sc2 = off;  off = align256(off + (size_t)T * 4);
    w.sg2 = off;  off = align256(off + (size_t)T * 4);
    w.total_without_splits = off;
    // the column splits' sums (one int per output of the larger stage, whole 256 x 64 blocks) and arrival counters
    w.slab = w.cnt = off;
    if (T <= SPLIT_MAX_T) {
        const size_t rg1 = (dbf_row_tiles(L->k) + QI_ROWTILES - 1) / QI_ROWTILES;
        const size_t rg2 = (dbf_row_tiles(L->n_out) + QI_ROWTILES - 1) / QI_ROWTILES;
        const size_t rg = rg1 > rg2 ? rg1 : rg2, tb = Tp / QI_TOKENS;
        off = align256(off + rg * tb * (QI_ROWTILES * DBF_TILE_ROWS) * QI_TOKENS * 4);
        w.cnt = off;  off = align256(off + rg * tb * 4 * SPLIT_CNT_STRIDE);
    }
    w.total = off;
    return w;
}

template <bool OUT_F32>
void launch_stage(StageArgs& s, unsigned tok_blocks, bool may_split, int* slab, unsigned* cnt, hipStream_t stream) {
    const int row_groups = (s.n_rt + QI_ROWTILES - 1) / QI_ROWTILES;
    s.splits = may_split ? pick_splits(row_groups, tok_blocks, s.n_ct) : 1;
    s.slab = slab;
    s.cnt = cnt;
    if (s.splits > 1)
        hipLaunchKernelGGL((dbf_gemm_i8_stage_kernel<OUT_F32, true>), dim3(row_groups, tok_blocks, s.splits), dim3(QI_THREADS), 0,
                           stream, s);
    else
        hipLaunchKernelGGL((dbf_gemm_i8_stage_kernel<OUT_F32, false>), dim3(row_groups, tok_blocks), dim3(QI_THREADS), 0, stream, s);
}

}  // namespace

size_t dbf_gemm_i8_workspace_bytes(const dbf_layer* L, int T) { return i8_workspace(L, T).total; }
size_t dbf_gemm_i8_workspace_bytes_without_splits(const dbf_layer* L, int T) { return i8_workspace(L, T).total_without_splits; }

// Launches quantise -> stage 1 -> quantise -> stage 2 on `stream`.  Arguments are validated by
// the caller (dbf_gemm); `ws` holds ws_bytes >= dbf_gemm_i8_workspace_bytes_without_splits(L, T) bytes; the stages
// of a call of few tokens cut their columns into shares if it also holds dbf_gemm_i8_workspace_bytes(L, T).
hipError_t dbf_gemm_i8_launch(const dbf_layer* L, const void* X_dev, void* Y_dev, int T, void* ws, size_t ws_bytes,
                              hipStream_t stream) {
    const I8Workspace w = i8_workspace(L, T);
    const bool may_split = T <= SPLIT_MAX_T && ws_bytes >= w.total;
    uint8_t* base = static_cast<uint8_t*>(ws);
    const int ks = dbf_row_tiles(L->k) * DBF_TILE_ROWS;
    const int kp1 = dbf_col_tiles(L->n_in) * DBF_TILE_COLS, kp2 = dbf_col_tiles(L->k) * DBF_TILE_COLS;
    const unsigned tok_blocks = (unsigned)((T + QI_TOKENS - 1) / QI_TOKENS);

    QuantArgs q1;
    q1.src = X_dev;  q1.col_scale = L->db;
    q1.dst = reinterpret_cast<signed char*>(base + w.xq1);
    q1.scale = reinterpret_cast<float*>(base + w.sc1);  q1.sigma = reinterpret_cast<int*>(base + w.sg1);
    q1.T = T;  q1.Tp = (T + 63) & ~63;  q1.cols = L->n_in;  q1.kp = kp1;  q1.ld = L->n_in;
    q1.vec_ok = ((L->n_in & 7) == 0 && (reinterpret_cast<uintptr_t>(X_dev) & 15) == 0) ? 1 : 0;
    q1.zero = may_split ? reinterpret_cast<v4u*>(base + w.slab) : nullptr;
    q1.zero_v4 = may_split ? (unsigned)((w.total - w.slab) / 16) : 0u;
    int* slab = reinterpret_cast<int*>(base + w.slab);
    unsigned* cnt = reinterpret_cast<unsigned*>(base + w.cnt);
    launch_quantise<false>(q1, kp1, T, stream);

    StageArgs s1;
    s1.bits = L->dB;  s1.row_scale = L->dm;
    s1.xq = q1.dst;  s1.scale = q1.scale;  s1.sigma = q1.sigma;
    s1.out = base + w.mid;
    s1.n_rt = dbf_row_tiles(L->k);  s1.n_ct = dbf_col_tiles(L->n_in);  s1.T = T;  s1.Tp = q1.Tp;  s1.ldo = ks;
    s1.n_valid = ks;  // padded rows have m = 0 and are written as zeros: the second quantisation reads them
    launch_stage<true>(s1, tok_blocks, may_split, slab, cnt, stream);

    QuantArgs q2;
    q2.src = base + w.mid;  q2.col_scale = nullptr;
    q2.dst = reinterpret_cast<signed char*>(base + w.xq2);
    q2.scale = reinterpret_cast<float*>(base + w.sc2);  q2.sigma = reinterpret_cast<int*>(base + w.sg2);
    q2.T = T;  q2.Tp = q1.Tp;  q2.cols = kp2 < ks ? kp2 : ks;  q2.kp = kp2;  q2.ld = ks;
    q2.vec_ok = 1;
    q2.zero = nullptr;  q2.zero_v4 = 0;
    launch_quantise<true>(q2, kp2, T, stream);

    StageArgs s2;
    s2.bits = L->dA;  s2.row_scale = L->da;
    s2.xq = q2.dst;  s2.scale = q2.scale;  s2.sigma = q2.sigma;
    s2.out = Y_dev;
    s2.n_rt = dbf_row_tiles(L->n_out);  s2.n_ct = dbf_col_tiles(L->k);  s2.T = T;  s2.Tp = q1.Tp;  s2.ldo = L->n_out;
    s2.n_valid = L->n_out;
    launch_stage<false>(s2, tok_blocks, may_split, slab, cnt, stream);
    return hipGetLastError();
}
