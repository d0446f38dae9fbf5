// Decode kernel with the int8 matrix cores as the adder.
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
// Work split: a workgroup (4 wavefronts) takes one item: `nrt` consecutive 128-row tiles of
// one stage of one layer; it quantises the input vector once for all of them.  Within a row
// tile wavefront w walks column tiles w, w+4, ... with PF tiles of sign bits in flight
// (buffer loads whose out-of-range lanes return zero, so the steady-state loop has no
// branches); the loads for the next row tile are already in flight while the current one is
// reduced.  The four partial results are added with integer LDS atomics (exact, order
// independent).  Between the prologue and the end of the item no load other than the
// sign-bit stream is issued (row scales are staged in LDS up front), so nothing drains the
// load pipeline.
//
// Fused launch: the item list holds every B-stage item before any A-stage item, and
// workgroups are dispatched in list order.  An A-stage workgroup waits (bounded) until the
// layer's B-stage workgroups have published all their rows of t, so both stages of all layers
// run in ONE launch and HBM never drains in between.  A B-stage workgroup never waits, so every
// wait ends; should the bound be hit anyway, the workgroup writes NaN to the outputs it owns
// and counts a time-out.  The counters only ever grow (no resets), so they stay consistent
// whatever happens: "published so far" is compared with what this launch must add on top of
// the launches that have completed.
#include <cstdlib>
#include <type_traits>

#include "dbf_kernels.h"
#include "dbf_wave.h"

// 1: tile loads by inline assembly with exact hand-placed waits (the fast path).
// 0: the same loads through the compiler builtin (it then waits with vmcnt(0) per group).
#ifndef DBF_ASM_LOADS
#define DBF_ASM_LOADS 1
#endif
// Cache-policy bits of the sign-bit loads.  Every sign bit is read exactly once per token, so
// the stream is marked non-temporal (measured: +10% over default-policy loads).
#ifndef DBF_LOAD_BITS
#define DBF_LOAD_BITS "nt"
#endif
#ifndef DBF_PROLOGUE_PRIO
#define DBF_PROLOGUE_PRIO 0
#endif
#ifndef DBF_PF
#define DBF_PF 4
#endif
#ifndef DBF_UNR
#define DBF_UNR 3
#endif
#ifndef DBF_WAVES_PER_EU
#define DBF_WAVES_PER_EU 4
#endif

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef unsigned short us8 __attribute__((ext_vector_type(8)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef unsigned int v6u __attribute__((ext_vector_type(6)));

constexpr int PF_DEFAULT = DBF_PF;  // tiles of sign bits kept in flight per wavefront
#ifndef DBF_PF_F4
#define DBF_PF_F4 4
#endif
#ifndef DBF_WAVES_F4
#define DBF_WAVES_F4 8
#endif
constexpr int WAVES_F4 = DBF_WAVES_F4;  // wavefronts per workgroup of the fp4 x bf6 form
constexpr int PF_F4 = DBF_PF_F4;    // the same in the fp4 x bf6 form, whose 48 KiB of operand rows leave room for two workgroups
                                    // per compute unit only: fewer wavefronts, each with more in flight
constexpr int UNR = DBF_UNR;       // independent 16-byte loads per thread in the prologue
constexpr int WIDE = 3;            // the same in the input passes of the kernel variant for wide rows and column pieces
constexpr float QMAX = 32512.f;    // 127*256: largest |q| so that hi and lo fit int8
constexpr int XQ_PAD = 16;         // bytes of padding per operand row (LDS bank spread)
#ifndef DBF_RB_STRIDE
#define DBF_RB_STRIDE 129
#endif
// Elements between operand columns of a reduction buffer: one more than the 128 rows of a tile, so that the
// lanes of a half wavefront (16 operand columns x 2 row groups) add into different LDS banks; with 128 all
// operand columns share a bank, which at 16 live columns (batch 8) made the reduction as long as the streaming.
constexpr int RB_STRIDE = DBF_RB_STRIDE;
constexpr unsigned OOB = 0x80000000u;  // buffer offset that is out of range for any span
// The fp4 x bf6 form of the operand (F4, batch 1): a stage input value q = d0 + 16 d1 + 256 d2 + 4096 d3 with signed hexadecimal
// digits (d0..d2 in -8..7, d3 in -8..8), each a bf6 (E3M2) number, which holds the integers up to 8 exactly.  LDS keeps eight
// operand rows: row p (0..3) has, per column, the pair (d_p, 0) of 6-bit fields, row 4 + p the pair (0, d_p) -- 12 bits per
// column, 96 bytes per column tile.  The pair lines up with the two nibbles of a sign byte (planes 0-3, planes 4-7).
// In LDS a column tile's 768 bytes are laid out word by word for the lanes that read them: lane (row r, 16-column group
// g) finds word k (0..5) of its 24 bytes at k * 128 + (4 r + g) * 4, so that every read instruction of a wavefront takes
// 32 different words from 32 different banks (with whole 24-byte runs per lane, however arranged, the reads cost
// three times their minimum in bank conflicts, and the LDS bounded the kernel).  A tile's block starts 784 bytes after
// the previous one's, which spreads the prologue's writes over the banks.
constexpr int F4_TILE_BYTES = 784;
constexpr int F4_MAX_COL_TILES = 64;   // 8 rows of 64 column tiles: 48 KiB, three workgroups per compute unit
constexpr uint16_t HALF_QNAN = 0x7E00; // what a workgroup that gave up its wait stores

__device__ inline float half_bits_to_float(uint16_t h) {
    return (float)__builtin_bit_cast(_Float16, h);
}
__device__ inline uint16_t float_to_half_bits(float f) {
    return __builtin_bit_cast(uint16_t, (_Float16)f);
}

// Fixed part of the LDS carve-up (the quantised operand and the reduction buffers follow).
struct Misc {
    float scale[DBF_MAX_BATCH];    // u ~= q * scale
    float inv[DBF_MAX_BATCH];      // q = rint(u * inv)
    int sigma[DBF_MAX_BATCH];      // sum over all columns of q
    float wmax[8][DBF_MAX_BATCH];  // per-wavefront max|u| (wavefronts 4-7, where a workgroup has them, take no part in
                                   // the input passes and leave zeros)
    uint16_t rscale[DBF_MAX_SPAN * DBF_TILE_ROWS];  // fp16 row scales of this workgroup's rows
    float out[DBF_MAX_SPAN * DBF_TILE_ROWS];        // batch 1, items of several row tiles: the finished rows, stored at the item's end
    int last;                      // column pieces: this workgroup was the last of its row tile to arrive
    int gave_up;                   // the wait for the layer's B stage ended at its bound: outputs become NaN
    int poisoned;                  // column pieces: some piece of this row tile gave up
    int pad_[1];
};
static_assert(sizeof(Misc) % 16 == 0, "the operand rows behind it are read in 16-byte pieces");

// Eight consecutive input values u[8*v .. 8*v+7] of batch row bi (vector item v).
// B stage: x (fp16) times b (fp16), exact in fp32.  A stage: the fp32 middle activations.
template <bool STAGE_A>
struct InputVec {
    v4u r0, r1;
    __device__ inline void load(const DbfItem& it, const uint16_t* x, int bi, int v, bool x_ok) {
        if (STAGE_A) {
            // t may have been written by another compute die during this very launch: read it
            // with agent-scope loads, which never return a stale line of this die's L2
            const unsigned* p = reinterpret_cast<const unsigned*>(it.t + (size_t)bi * it.t_stride) + 8 * (size_t)v;
            r0.x = __hip_atomic_load(p + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r0.y = __hip_atomic_load(p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r0.z = __hip_atomic_load(p + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r0.w = __hip_atomic_load(p + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r1.x = __hip_atomic_load(p + 4, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r1.y = __hip_atomic_load(p + 5, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r1.z = __hip_atomic_load(p + 6, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            r1.w = __hip_atomic_load(p + 7, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else {
            r1 = __builtin_bit_cast(v4u, reinterpret_cast<const us8*>(it.in_scale)[v]);
            r0 = (v4u){0, 0, 0, 0};
            if (x_ok) r0 = __builtin_bit_cast(v4u, reinterpret_cast<const us8*>(x + (size_t)bi * it.cols)[v]);
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
    __device__ inline float absmax() const {
        float u[8], m = 0.f;
        get(u);
#pragma unroll
        for (int i = 0; i < 8; ++i) m = fmaxf(m, fabsf(u[i]));
        return m;
    }
    // Quantises the eight values, stores the two int8 planes, returns the sum of the q.
    // q = 256 hi + lo with lo in [-128, 127]: with t = q + 128, hi is byte 1 of t (t >> 8, sign included,
    // |q| <= 32512) and lo is byte 0 of t with its top bit flipped (t mod 256 - 128).  The bytes of the
    // eight t are gathered with byte permutes: one for two values, then one per plane for four.
    __device__ inline int quantise_to(signed char* hi_dst, signed char* lo_dst, float inv) const {
        float u[8];
        get(u);
        unsigned pair[4];
        int sum = 0;
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            const int q0 = (int)__builtin_amdgcn_fmed3f(rintf(u[i] * inv), -QMAX, QMAX);
            const int q1 = (int)__builtin_amdgcn_fmed3f(rintf(u[i + 1] * inv), -QMAX, QMAX);
            sum += q0 + q1;
            // bytes (t0.b0, t1.b0, t0.b1, t1.b1); selector bytes 0-3 pick from the second source, 4-7 from the first
            pair[i >> 1] = __builtin_amdgcn_perm((unsigned)(q1 + 128), (unsigned)(q0 + 128), 0x05010400u);
        }
        unsigned hi4[2], lo4[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            lo4[h] = __builtin_amdgcn_perm(pair[2 * h + 1], pair[2 * h], 0x05040100u) ^ 0x80808080u;
            hi4[h] = __builtin_amdgcn_perm(pair[2 * h + 1], pair[2 * h], 0x07060302u);
        }
        *reinterpret_cast<uint2*>(hi_dst) = make_uint2(hi4[0], hi4[1]);
        *reinterpret_cast<uint2*>(lo_dst) = make_uint2(lo4[0], lo4[1]);
        return sum;
    }
    // The same eight q as signed hexadecimal digits in bf6, into the eight operand rows of the fp4 x bf6 form (row r at
    // the words the lanes of the matrix instruction read, see F4_TILE_BYTES); returns the sum of the q.  The conversion
    // instruction takes two vectors of 16 floats and interleaves them: (digits, zeros) gives the pairs (d, 0) of two rows
    // -- eight columns of digit plane p in elements 0-7, of plane p + 1 in elements 8-15 -- and (zeros, digits) the pairs (0, d).
    __device__ inline int quantise_f4(signed char* dst, float inv) const {
        float u[8];
        get(u);
        v16f d01, d23;
        int sum = 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int q = (int)__builtin_amdgcn_fmed3f(rintf(u[i] * inv), -QMAX, QMAX);
            sum += q;
            const int q1 = (q + 8) >> 4, q2 = (q1 + 8) >> 4;  // (the extract below is signed; the builtin's type is not)
            d01[i] = (float)(int)__builtin_amdgcn_sbfe(q, 0, 4);
            d01[8 + i] = (float)(int)__builtin_amdgcn_sbfe(q1, 0, 4);
            d23[i] = (float)(int)__builtin_amdgcn_sbfe(q2, 0, 4);
            d23[8 + i] = (float)((q2 + 8) >> 4);
        }
        v16f zero;
#pragma unroll
        for (int i = 0; i < 16; ++i) zero[i] = 0.f;
        const v6u lo01 = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(d01, zero, 1.0f);
        const v6u lo23 = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(d23, zero, 1.0f);
        const v6u hi01 = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(zero, d01, 1.0f);
        const v6u hi23 = __builtin_amdgcn_cvt_scalef32_2xpk16_bf6_f32(zero, d23, 1.0f);
        // (dst: word 0 of row 0 for this item's 16-column group; its eight columns are three of the group's six words)
        auto put = [&](int row, unsigned a, unsigned b, unsigned c) {
            unsigned* o = reinterpret_cast<unsigned*>(dst) + 4 * row;
            o[0] = a;  o[32] = b;  o[64] = c;
        };
        put(0, lo01[0], lo01[1], lo01[2]);  put(1, lo01[3], lo01[4], lo01[5]);
        put(2, lo23[0], lo23[1], lo23[2]);  put(3, lo23[3], lo23[4], lo23[5]);
        put(4, hi01[0], hi01[1], hi01[2]);  put(5, hi01[3], hi01[4], hi01[5]);
        put(6, hi23[0], hi23[1], hi23[2]);  put(7, hi23[3], hi23[4], hi23[5]);
        return sum;
    }
};

template <bool STAGE_A>
__device__ inline float load_u_scalar(const DbfItem& it, const uint16_t* x, int bi, int l) {
    if (STAGE_A)
        return __builtin_bit_cast(float, __hip_atomic_load(reinterpret_cast<const unsigned*>(it.t) + (size_t)bi * it.t_stride + l,
                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    return half_bits_to_float(x[(size_t)bi * it.cols + l]) * half_bits_to_float(it.in_scale[l]);
}

// What the input helpers need to know about the workgroup.
struct Ctx {
    Misc* misc;
    signed char* xq;
    const uint16_t* x;  // B stage input rows (fp16), unused in the A stage
    int chs;            // bytes from the high plane of a batch row to its low plane (LDS: the operand row's length)
    int tstride;        // TILED destinations only: bytes from one column tile of a plane to the next
    int tid, lane, w;
    int batch;
    bool fast;          // 16-byte vector loads are possible
    int nvec, nvec_x;   // vector items per row incl. padding / items backed by x
};

// The decode case in one pass: the row was loaded once into registers (by the kernel's
// prologue, see there); reduce max|u| and quantise from the registers.
// Contains one barrier; ends with the operand in LDS (not yet synchronised).
// TILED: the destination is not an LDS operand row but the per-call buffer of a stage (DbfStage::q_in), in which
// the 64 bytes a plane has for one column tile are followed by the next plane's.
template <bool STAGE_A, bool TILED = false>
__device__ inline void input_one_pass(const Ctx& c, const v4u (&r0)[UNR], const v4u (&r1)[UNR]) {
    InputVec<STAGE_A> iv[UNR];
    float mx = 0.f;
#pragma unroll
    for (int j = 0; j < UNR; ++j) {
        const int v = 256 * j + c.tid;
        iv[j].r0 = (STAGE_A || v < c.nvec_x) ? r0[j] : (v4u){0, 0, 0, 0};  // beyond x the product is zero
        iv[j].r1 = r1[j];
    }
#pragma unroll
    for (int j = 0; j < UNR; ++j)
        if (256 * j + c.tid < c.nvec) mx = fmaxf(mx, iv[j].absmax());
    mx = dbf_wave_max(mx);
    if (c.lane == 0) c.misc->wmax[c.w][0] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(c.misc->wmax[0][0], c.misc->wmax[1][0]), fmaxf(c.misc->wmax[2][0], c.misc->wmax[3][0]));
    const float inv = mx > 0.f ? QMAX / mx : 0.f;
    if (c.tid == 0) c.misc->scale[0] = mx / QMAX;
    int local = 0;
#pragma unroll
    for (int j = 0; j < UNR; ++j) {
        const int v = 256 * j + c.tid;
        const int at = TILED ? (v >> 3) * c.tstride + (v & 7) * 8 : v * 8;
        if (v < c.nvec) local += iv[j].quantise_to(c.xq + at, c.xq + c.chs + at, inv);
    }
    local = dbf_wave_sum(local);
    if (c.lane == 0) atomicAdd(&c.misc->sigma[0], local);
}

// The same for the fp4 x bf6 form: all T threads of the workgroup take part, one vector item each (rows of up to 8 T
// values), and the destination is the eight-row digit form.
template <bool STAGE_A, int T>
__device__ inline void input_one_pass_f4(const Ctx& c, const v4u& r0, const v4u& r1) {
    InputVec<STAGE_A> iv;
    const int v = c.tid;
    iv.r0 = (STAGE_A || v < c.nvec_x) ? r0 : (v4u){0, 0, 0, 0};  // beyond x the product is zero
    iv.r1 = r1;
    float mx = v < c.nvec ? iv.absmax() : 0.f;
    mx = dbf_wave_max(mx);
    if (c.lane == 0) c.misc->wmax[c.w][0] = mx;
    __syncthreads();
    mx = 0.f;
#pragma unroll
    for (int i = 0; i < T / 64; ++i) mx = fmaxf(mx, c.misc->wmax[i][0]);
    const float inv = mx > 0.f ? QMAX / mx : 0.f;
    if (c.tid == 0) c.misc->scale[0] = mx / QMAX;
    int local = 0;
    // (vector item v: column tile v >> 3, 16-column group (v & 7) >> 1, first or second half of that group's six words)
    if (v < c.nvec) local = iv.quantise_f4(c.xq + (v >> 3) * F4_TILE_BYTES + 4 * ((v & 7) >> 1) + 384 * (v & 1), inv);
    local = dbf_wave_sum(local);
    if (c.lane == 0) atomicAdd(&c.misc->sigma[0], local);
}

// General case, first pass: max|u| of every batch row -> scale / inv.  Two barriers.
template <bool STAGE_A, int W>
__device__ inline void input_scales(const DbfItem& it, const Ctx& c) {
    for (int bi = 0; bi < c.batch; ++bi) {
        float mx = 0.f;
        if (c.fast) {
            // (W vector items per thread and round: all their loads are in flight together, so a
            // wide row costs a few memory latencies, not one per 256*W*8 columns)
            for (int base = 0; base < c.nvec; base += 256 * W) {
                InputVec<STAGE_A> iv[W];
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    const int v = base + 256 * j + c.tid;
                    if (v < c.nvec) iv[j].load(it, c.x, bi, v, v < c.nvec_x);
                }
#pragma unroll
                for (int j = 0; j < W; ++j)
                    if (base + 256 * j + c.tid < c.nvec) mx = fmaxf(mx, iv[j].absmax());
            }
        } else {
            for (int l = c.tid; l < it.cols; l += 256) mx = fmaxf(mx, fabsf(load_u_scalar<STAGE_A>(it, c.x, bi, l)));
        }
        mx = dbf_wave_max(mx);
        if (c.lane == 0) c.misc->wmax[c.w][bi] = mx;
    }
    __syncthreads();
    if (c.tid < c.batch) {
        const float mx = fmaxf(fmaxf(c.misc->wmax[0][c.tid], c.misc->wmax[1][c.tid]),
                               fmaxf(c.misc->wmax[2][c.tid], c.misc->wmax[3][c.tid]));
        c.misc->scale[c.tid] = mx / QMAX;
        c.misc->inv[c.tid] = mx > 0.f ? QMAX / mx : 0.f;
    }
    __syncthreads();
}

// General case, second pass: quantise columns [64*c0, 64*cend) of every batch row into LDS.
template <bool STAGE_A, int W, bool TILED = false>
__device__ inline void input_quantise_chunk(const DbfItem& it, const Ctx& c, int c0, int cend) {
    for (int bi = 0; bi < c.batch; ++bi) {
        const float inv = c.misc->inv[bi];
        int local = 0;
        signed char* hi_row = c.xq + (2 * bi) * c.chs;
        signed char* lo_row = c.xq + (2 * bi + 1) * c.chs;
        if (c.fast) {
            const int v0 = c0 * 8, v1 = cend * 8;
            for (int base = v0; base < v1; base += 256 * W) {
                InputVec<STAGE_A> iv[W];
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    const int v = base + 256 * j + c.tid;
                    if (v < v1) iv[j].load(it, c.x, bi, v, v < c.nvec_x);
                }
#pragma unroll
                for (int j = 0; j < W; ++j) {
                    const int v = base + 256 * j + c.tid;
                    const int at = TILED ? ((v - v0) >> 3) * c.tstride + ((v - v0) & 7) * 8 : (v - v0) * 8;
                    if (v < v1) local += iv[j].quantise_to(hi_row + at, lo_row + at, inv);
                }
            }
        } else {
            for (int l = c0 * 64 + c.tid; l < cend * 64; l += 256) {
                int q = 0;
                if (l < it.cols) {
                    float f = rintf(load_u_scalar<STAGE_A>(it, c.x, bi, l) * inv);
                    f = fminf(fmaxf(f, -QMAX), QMAX);
                    q = (int)f;
                }
                const int lo = ((q + 128) & 255) - 128;
                const int hi = (q - lo) >> 8;
                const int rel = l - c0 * 64;
                const int at = TILED ? (rel >> 6) * c.tstride + (rel & 63) : rel;
                hi_row[at] = (signed char)hi;
                lo_row[at] = (signed char)lo;
                local += q;
            }
        }
        local = dbf_wave_sum(local);
        if (c.lane == 0) atomicAdd(&c.misc->sigma[bi], local);
    }
}

// PIECES: the variant for lists whose items may be column pieces of a row tile (few row tiles) or
// have rows too wide for the one-pass prologue; its input passes keep more loads in flight.  The
// other instantiation is the hot one (long streams of layers of up to 4096 columns at batch 1)
// and carries none of that code.
// SHARED != 0: the stage input was quantised once for the whole launch by dbf_quantise_inputs_kernel (batches
// of 2 and more, where every item quantising all batch rows itself would cost more than streaming its tiles;
// stacks of layers with long stage inputs at batch 1 too): the prologue takes scales and sums from there.
// SHARED == 1: the int8 planes of the item's columns are copied into LDS and read from there as at batch 1.
// SHARED == 2 (rows that do not fit the LDS of a workgroup at this batch): no operand in LDS at all; the 16
// operand bytes a lane needs for a tile are requested from memory (the planes are L2 resident: every item of
// the layer reads them) together with the tile, in the same ring.  SHARED == 3: as 2, but every wavefront takes
// a row tile of its own and all four walk the same column tiles together, so that their operand reads meet in
// the compute unit's vector cache (lists of long items: what streams take at batch 2 and more).
// SINGLE: every item of the launch streams its columns as one chunk (the launcher knows): the first group of
// tiles of a row tile then starts from zero accumulators by giving the matrix instructions a zero addend,
// and the 32 accumulator registers are never cleared (2 of 47 vector instructions per tile).
// WAVES: wavefronts per workgroup.  Eight for launches of so few items that a compute unit gets one workgroup at
// most (a layer alone, a group of three): a wavefront then walks every eighth column tile of a row tile instead of
// every fourth, and two wavefronts per SIMD fill each other's waits.  Wavefronts 4-7 only stream tiles: the input
// passes and the epilogue are those of the four-wavefront kernel, done by threads 0-255.
// F4 (batch 1, rows of up to 4096 columns that take the one-pass prologue): the sign operand goes to the matrix cores as
// fp4 and the stage input as bf6 digits, v_mfma_f32_16x16x128_f8f6f4.  A nibble mask over a tile's bytes makes TWO bit
// planes an operand at once (the two nibbles of a byte are neighbouring K slots; the input rows (d, 0) and (0, d) send
// them to different output columns), so a tile costs 4 matrix instructions of 4 passes and 20 vector instructions
// instead of 8 and 32.  The sums are integers below 2^24 in fp32: exact, and the result is bit for bit that of the
// int8 form.
template <int NCG, bool PIECES, int SHARED, bool SINGLE, int WAVES = 4, bool F4 = false>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(NCG == 1 ? DBF_WAVES_PER_EU : 2)))
void dbf_items_mfma_kernel(const DbfItem* __restrict__ items, unsigned long long* __restrict__ sync, int n_layers,
                           int use_sync, const uint16_t* __restrict__ x_base,
                           uint16_t* __restrict__ y_base, int batch, int ch_tiles, int wait_limit_us) {
    static_assert(WAVES == 4 || (WAVES == 8 && SHARED == 0 && !PIECES), "eight wavefronts: self-quantising whole-row items only");
    static_assert(!F4 || (NCG == 1 && !PIECES && SHARED == 0 && SINGLE), "fp4 x bf6: batch 1, whole rows in one chunk");
    constexpr int PF = F4 ? PF_F4 : PF_DEFAULT;
    extern __shared__ __align__(16) unsigned char smem[];
    const int ncols = 2 * batch;
    const int chs = F4 ? 16 : ch_tiles * DBF_TILE_COLS + XQ_PAD;  // (F4: row r of a tile's block starts at word 4 r)
    Misc* misc = reinterpret_cast<Misc*>(smem);
    signed char* xq = reinterpret_cast<signed char*>(smem + sizeof(Misc));           // [ncols][chs]
    // RING: the operand comes from memory with the tile (SHARED 2 and 3).  ROWS (SHARED 3): the four wavefronts
    // do not share a row tile's column tiles but take a row tile each, all of them walking the same columns at
    // the same time -- so three of the four reads of an operand hit the compute unit's first-level cache --
    // and reduce into a buffer of their own.
    constexpr bool RING = SHARED >= 2, ROWS = SHARED == 3;
    constexpr int N_RED = ROWS ? 4 : 2;  // reduction buffers
    constexpr int RT_STEP = ROWS ? 4 : 1;  // row tiles the workgroup works on at a time
    int* red = reinterpret_cast<int*>(smem + sizeof(Misc) + (RING ? 0 : F4 ? ch_tiles * F4_TILE_BYTES : ((ncols * chs + 15) & ~15)));  // [N_RED][ncols][128]

#if DBF_PROLOGUE_PRIO
    // (experiment: wavefront priority raised for the prologue.  The arbiter favours older
    // wavefronts, so the youngest workgroup's prologue is slow -- but what it gains the streaming
    // neighbours lose; measured neutral, left off.)
    __builtin_amdgcn_s_setprio(DBF_PROLOGUE_PRIO);
#endif
    constexpr int IN_W = PIECES ? WIDE : UNR;
    const DbfItem it = items[blockIdx.x];
    // Fields only the epilogue of a column piece needs are read again there instead of living in scalar
    // registers through the whole kernel (the volatile asm keeps the compiler from merging the reads).
    auto late = [&]() { const DbfItem* q = items + blockIdx.x; asm volatile("" : "+s"(q)); return q; };
    auto piece_acc = [&]() { return late()->acc; };
    auto piece_cnt = [&]() { return late()->cnt; };
    auto piece_acc_stride = [&]() { return late()->acc_stride; };
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const bool stage_a = it.stage_a != 0;
    const uint16_t* x = x_base + it.io_off * batch;  // B stage only
    uint16_t* y = y_base + it.io_off * batch;        // A stage only

    // sign bits of this item's row tiles: one contiguous span, addressed through a buffer
    // resource so that out-of-range offsets read as zero without touching memory
    const uint64_t span_addr = reinterpret_cast<uint64_t>(it.bits);
    v4u rsrc;  // raw buffer descriptor: base, stride 0, size in bytes, 32-bit raw data format
    rsrc.x = __builtin_amdgcn_readfirstlane((unsigned)span_addr);
    rsrc.y = __builtin_amdgcn_readfirstlane((unsigned)(span_addr >> 32) & 0xFFFFu);
    rsrc.z = __builtin_amdgcn_readfirstlane((unsigned)(it.nrt * it.n_ct * DBF_TILE_BYTES));
    rsrc.w = 0x00020000u;
    const unsigned lane_off = lane * 16;

    // Tile cursor of the prefetcher: row tile p_rt (local), step p_i of the chunk.  Step i of a
    // wavefront is column tile c0 + w + WAVES*i; steps are padded to a multiple of PF per row tile.
    //
    // The loads are issued by inline assembly and waited for by hand (wait_slot): the compiler
    // does not see them, so it cannot serialise the pipeline with a full vmcnt(0) wait at the
    // top of the loop.  Loads complete in issue order; when slot j is consumed exactly PF-1
    // younger tile loads are outstanding, so vmcnt(PF-1) is the exact wait.  Any other memory
    // operation the compiler issues in between only makes that wait more conservative.
    // (An item covers column tiles [ct0, ct_end) of its row tiles: all of them, unless the row tile is
    // cut into column pieces.)
    const int ct_first = PIECES ? it.ct0 : 0;
    const int ct_end = PIECES ? it.ct0 + it.ct_n : it.n_ct;
    const int n_pieces = PIECES ? it.pieces : 1;
    int c0 = ct_first;
    int cend = min(ct_end, c0 + ch_tiles);
    // (steps of a wavefront per row tile and chunk: every WAVES-th column tile, or with ROWS every one)
    auto steps_of = [&](int n_tiles) { return ((ROWS ? n_tiles : (n_tiles + WAVES - 1) / WAVES) + PF - 1) / PF * PF; };
    int steps = steps_of(cend - c0);
    int p_rt = 0, p_i = 0;  // (ROWS: p_rt counts groups of four row tiles, of which this wavefront takes the w-th)
    v4u buf[PF];
    // SHARED == 2: the operand ring.  A second buffer resource covers the 2 * batch planes of the stage, laid out
    // column tile by column tile (per tile: plane 0's 64 bytes, plane 1's, ...), so that what a wavefront reads for a
    // tile is one contiguous run of 64 * 2 * batch bytes; lane (g, c) of column group gi reads bytes 16 g .. 16 g +
    // 15 of plane 16 gi + c (unused operand columns alias a valid plane).  A slot's loads are issued as (tile,
    // operand[0], operand[1]).  (With whole plane rows one after the other every lane of a load touched a cache
    // line of its own: 8 KiB moved from the L2 per 1 KiB used, and that traffic bounded batches 5-16.)
    constexpr int XB_N = RING ? NCG : 1;
    constexpr int SLOT_LOADS = RING ? 1 + NCG : 1;
    v4i xb[PF][XB_N];
    v4u xrsrc = {0, 0, 0, 0};
    unsigned x_lane_off[XB_N] = {};
    if (RING) {
        const uint64_t pa = reinterpret_cast<uint64_t>(it.q_in + DBF_QIN_HEADER);
        xrsrc.x = __builtin_amdgcn_readfirstlane((unsigned)pa);
        xrsrc.y = __builtin_amdgcn_readfirstlane((unsigned)(pa >> 32) & 0xFFFFu);
        xrsrc.z = __builtin_amdgcn_readfirstlane((unsigned)(ncols * it.n_ct * DBF_TILE_COLS));
        xrsrc.w = 0x00020000u;
#pragma unroll
        for (int gi = 0; gi < XB_N; ++gi) {
            const int col = 16 * gi + c;
            x_lane_off[gi] = (unsigned)((col < ncols ? col : col % ncols) * DBF_TILE_COLS + 16 * g);
        }
    }
    auto fetch_operand = [&](int j, int ct, int ok) {
        if (RING) {
#pragma unroll
            for (int gi = 0; gi < XB_N; ++gi) {
                const unsigned voff = ok ? x_lane_off[gi] + (unsigned)(ct * ncols) * DBF_TILE_COLS : OOB;
                asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen" : "=v"(xb[j][gi]) : "v"(voff), "s"(xrsrc) : "memory");
            }
        }
    };
    // (the load itself, for a tile at byte offset `off` of the item's span; !ok: a placeholder that returns zeros)
    auto fetch_at = [&](int j, unsigned off, int ct, int ok) {
        v4u& dst = buf[j];
        const unsigned voff = lane_off + (ok ? off : OOB);
#if DBF_ASM_LOADS
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen " DBF_LOAD_BITS
                     : "=v"(dst) : "v"(voff), "s"(rsrc) : "memory");
#else
        dst = __builtin_amdgcn_raw_buffer_load_b128(
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(it.bits), 0, (int)rsrc.z, 0x00020000),
            voff, 0, 0);
#endif
        fetch_operand(j, ct, ok);
    };
    auto fetch = [&](int j) {
        v4u& dst = buf[j];
        const int ct = ROWS ? c0 + p_i : c0 + w + WAVES * p_i;
        const int rt = ROWS ? 4 * p_rt + w : p_rt;
        const int ok = (int)(rt < it.nrt) & (int)(ct < cend);
        const unsigned off = (unsigned)(rt * it.n_ct + ct) * DBF_TILE_BYTES;
        const unsigned voff = lane_off + (ok ? off : OOB);
#if DBF_ASM_LOADS
        asm volatile("buffer_load_dwordx4 %0, %1, %2, 0 offen " DBF_LOAD_BITS
                     : "=v"(dst) : "v"(voff), "s"(rsrc) : "memory");
#else
        dst = __builtin_amdgcn_raw_buffer_load_b128(
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t*>(it.bits), 0, (int)rsrc.z, 0x00020000),
            voff, 0, 0);
#endif
        fetch_operand(j, ct, ok);
        const int wrap = (int)(p_i + 1 == steps);
        p_i = wrap ? 0 : p_i + 1;
        p_rt += wrap;
    };
    auto wait_slot = [&](int j) {
#if DBF_ASM_LOADS
        if (RING && NCG == 2)
            asm volatile("s_waitcnt vmcnt(%3)" : "+v"(buf[j]), "+v"(xb[j][0]), "+v"(xb[j][XB_N - 1]) : "n"((PF - 1) * SLOT_LOADS) : "memory");
        else if (RING)
            asm volatile("s_waitcnt vmcnt(%2)" : "+v"(buf[j]), "+v"(xb[j][0]) : "n"((PF - 1) * SLOT_LOADS) : "memory");
        else
            asm volatile("s_waitcnt vmcnt(%1)" : "+v"(buf[j]) : "n"(PF - 1) : "memory");
#endif
    };
    auto retire_ring = [&]() {
#if DBF_ASM_LOADS
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
        for (int j = 0; j < PF; ++j) {
            asm volatile("" : "+v"(buf[j]));
            if (RING) {
#pragma unroll
                for (int gi = 0; gi < XB_N; ++gi) asm volatile("" : "+v"(xb[j][gi]));
            }
        }
#endif
    };
    // ---- fused launch: an A-stage item waits for the layer's B stage ---------------------
    // (Counter i is sync[i * DBF_SYNC_STRIDE]: 512 bytes apart, so that the workgroups polling different layers'
    // counters do not all queue at one memory channel.)
    // sync[layer] counts the B-stage row tiles published over all one-launch calls of this plan, sync[n_layers +
    // layer] the A-stage row tiles finished: what one call adds to either (it.need, it.peers: the layer's B and A
    // row tiles) does not depend on how the call's list cuts the layer into items, so calls may switch lists.
    // Launches of one plan do not overlap, so while this launch runs the second counter lies in [e * peers,
    // (e + 1) * peers) with e the number of completed launches, and this launch's B stage is done when the first
    // counter has reached (e + 1) * need.  The wait is bounded on the GPU's constant 100 MHz clock.
    if (tid == 0) misc->gave_up = 0;
    if (use_sync && stage_a) {
        if (tid == 0) {
            const unsigned long long fin = __hip_atomic_load(&sync[(size_t)(n_layers + it.layer) * DBF_SYNC_STRIDE], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            const unsigned long long target = (fin / (unsigned)it.peers + 1ull) * (unsigned)it.need;
            const unsigned long long t0 = __builtin_amdgcn_s_memrealtime();
            const unsigned long long limit = 100ull * (unsigned)wait_limit_us;
            while (__hip_atomic_load(&sync[(size_t)it.layer * DBF_SYNC_STRIDE], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < target) {
                if (__builtin_amdgcn_s_memrealtime() - t0 >= limit) {  // never expected; keeps every wave finite
                    __hip_atomic_fetch_add(&sync[(size_t)(2 * n_layers) * DBF_SYNC_STRIDE], 1ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    misc->gave_up = 1;
                    break;
                }
                __builtin_amdgcn_s_sleep(16);
            }
        }
        __syncthreads();  // t is read below with agent-scope loads, so no cache invalidation is needed
    }

    // ---- prologue ------------------------------------------------------------------------------
    Ctx cx;
    cx.misc = misc;  cx.xq = xq;  cx.x = x;  cx.chs = chs;  cx.tstride = 0;
    // (wavefronts 4-7 of an eight-wavefront workgroup stream tiles only.  For the input passes they get a thread index
    //  beyond every range those test, so they only keep the barriers company; of the prologue's loads they issue
    //  the tiles alone -- its wait counts back from the youngest load)
    const bool streams_only = WAVES > 4 && !F4 && tid >= 256;  // (F4: every thread has a vector item of the input)
    constexpr int IN_T = F4 ? 64 * WAVES : 256;  // threads that take part in the input passes ...
    constexpr int IN_U = F4 ? 1 : UNR;           // ... and vector items each of them holds in the one-pass prologue
    cx.tid = streams_only ? (1 << 28) : tid;  cx.lane = lane;  cx.w = w;  cx.batch = batch;
    cx.nvec = it.n_ct * 8;
    cx.nvec_x = it.cols >> 3;
    cx.fast = stage_a || ((it.cols & 7) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0);
    const bool one_pass = !SHARED && cx.fast && batch == 1 && cx.nvec <= IN_T * IN_U && it.n_ct <= ch_tiles;

    // Every load of the prologue is issued here, back to back and in order of urgency: the row
    // scales and the input vector FIRST (the workgroup cannot start without them), then the first
    // PF sign tiles.  Loads complete in issue order, so the small critical loads do not queue
    // behind 4 KiB of tiles per wavefront, and one wait that leaves the PF youngest loads (the
    // tiles) in flight covers them.  All of it is straight-line inline assembly with every
    // destination named by the wait: addresses are clamped instead of branching, and whatever a
    // lane loaded beyond its range is ignored later.  (The general path below does not use the
    // input registers; for it the loads are merely harmless.)
    constexpr int RS_WORDS = DBF_MAX_SPAN * DBF_TILE_ROWS / 2 / IN_T;
    unsigned rs_reg[RS_WORDS];
    v4u in0[UNR], in1[UNR];
    if (!streams_only) {
        const int rs_last = it.nrt * (DBF_TILE_ROWS / 2) - 1;
#pragma unroll
        for (int q = 0; q < RS_WORDS; ++q) {
            const unsigned* p = reinterpret_cast<const unsigned*>(it.row_scale) + min(tid + IN_T * q, rs_last);
            asm volatile("global_load_dword %0, %1, off" : "=v"(rs_reg[q]) : "v"(p) : "memory");
        }
#pragma unroll
        for (int j = 0; j < IN_U; ++j) {
            const int v = min(IN_T * j + tid, cx.nvec - 1);
            const int vx = max(min(v, cx.nvec_x - 1), 0);
            // A stage: 8 fp32 of t (agent scope: maybe written by another compute die during this
            // launch).  B stage: 8 fp16 of x and of b; if x cannot be read in 16-byte pieces
            // the general path is taken and b stands in for it here.
            const void* p0 = stage_a ? static_cast<const void*>(it.t + 8 * (size_t)v)
                                     : (cx.fast ? static_cast<const void*>(x + 8 * (size_t)vx)
                                                : static_cast<const void*>(it.in_scale + 8 * (size_t)v));
            const void* p1 = stage_a ? static_cast<const void*>(it.t + 8 * (size_t)v + 4)
                                     : static_cast<const void*>(it.in_scale + 8 * (size_t)v);
            asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(in0[j]) : "v"(p0) : "memory");
            asm volatile("global_load_dwordx4 %0, %1, off sc1" : "=v"(in1[j]) : "v"(p1) : "memory");
        }
    }
#pragma unroll
    for (int j = 0; j < PF; ++j) fetch(j);
#if DBF_ASM_LOADS
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(PF * SLOT_LOADS) : "memory");
#else
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#endif
#pragma unroll
    for (int q = 0; q < RS_WORDS; ++q) asm volatile("" : "+v"(rs_reg[q]));
#pragma unroll
    for (int j = 0; j < IN_U; ++j) asm volatile("" : "+v"(in0[j]), "+v"(in1[j]));

    const int rcols = F4 ? 4 : ncols;  // operand columns of a reduction buffer (F4: the four digits)
    for (int i = tid; i < N_RED * RB_STRIDE * rcols; i += 64 * WAVES) red[i] = 0;
    if (tid < DBF_MAX_BATCH) misc->sigma[tid] = 0;
    // row scales: read by the epilogues, which come after several barriers
#pragma unroll
    for (int q = 0; q < RS_WORDS; ++q) {
        const int idx = tid + IN_T * q;
        if (!streams_only && 2 * idx < it.nrt * DBF_TILE_ROWS) reinterpret_cast<unsigned*>(misc->rscale)[idx] = rs_reg[q];
    }

    if (SHARED) {
        if (tid < batch) {  // (the same threads that cleared sigma above)
            misc->scale[tid] = reinterpret_cast<const float*>(it.q_in)[tid];
            misc->sigma[tid] = reinterpret_cast<const int*>(it.q_in + 64)[tid];
        }
    } else if (one_pass && F4) {
        if (stage_a) input_one_pass_f4<true, IN_T>(cx, in0[0], in1[0]); else input_one_pass_f4<false, IN_T>(cx, in0[0], in1[0]);
    } else if (one_pass) {
        if (stage_a) input_one_pass<true>(cx, in0, in1); else input_one_pass<false>(cx, in0, in1);
    } else if (F4) {
        // (the launcher takes this form only for launches whose rows all take the one-pass prologue; should one not, its
        //  outputs say so like those of a wait that gave up)
        if (tid == 0) misc->gave_up = 1;
    } else {
        if (stage_a) input_scales<true, IN_W>(it, cx); else input_scales<false, IN_W>(it, cx);
    }

    v4i acc[NCG][8];
    v4f accf[4];  // F4: sums of bit planes s and 4 + s (operand columns 0-3 and 4-7: the four digits)
    // operand row this lane feeds to the matrix instruction (unused columns alias a valid row)
    int xrow[NCG];
#pragma unroll
    for (int gi = 0; gi < NCG; ++gi) {
        const int col = 16 * gi + c;
        xrow[gi] = F4 ? (c & 7) * chs + 4 * g : (col < ncols ? col : col % ncols) * chs + 16 * g;
    }
    // one pass: the whole row is in LDS at its own column offsets; otherwise LDS holds the current chunk
    constexpr int X_TILE = F4 ? F4_TILE_BYTES : DBF_TILE_COLS;  // operand bytes per column tile and row
    const int xo_base = one_pass ? ct_first * X_TILE : 0;
    // epilogue coordinates: thread -> (row rho of the tile, batch rows bi = tid>>7, +2, ...)
    const int rho = tid & 127;
    const int e_s = rho >> 4;
    int tile_no = 0;  // row tiles finished so far: selects the reduction buffer
    // batch 1, whole rows in one chunk: finished rows wait in LDS for the end of the item (see the epilogue)
    const bool defer = SINGLE && SHARED == 0 && !PIECES && batch == 1;

#if DBF_PROLOGUE_PRIO
    __builtin_amdgcn_s_setprio(0);
#endif
    // The accumulators start at zero and are cleared again right after every reduction (unconditionally: a
    // conditional clear at the top of a row tile becomes 32 selects or 64 register copies).
#pragma unroll
    for (int gi = 0; gi < NCG; ++gi)
#pragma unroll
        for (int s = 0; s < 8; ++s) acc[gi][s] = (v4i){0, 0, 0, 0};
#pragma unroll
    for (int s = 0; s < 4; ++s) accf[s] = (v4f){0.f, 0.f, 0.f, 0.f};
    for (;;) {  // chunks of columns (a single one unless the batch is large)
        if (SHARED == 1) {
            // columns [64 c0, 64 cend) of the 2 * batch planes, 16 bytes per thread and round
            // (in the buffer the planes alternate column tile by column tile; in LDS every plane is one row)
            const unsigned char* planes = it.q_in + DBF_QIN_HEADER + (size_t)c0 * ncols * DBF_TILE_COLS;
            const int per_row = (cend - c0) * (DBF_TILE_COLS / 16);
            for (int r = 0; r < ncols; ++r)
                for (int i = tid; i < per_row; i += 256)
                    *reinterpret_cast<v4u*>(xq + r * chs + 16 * i) = *reinterpret_cast<const v4u*>(
                        planes + ((size_t)(i >> 2) * ncols + r) * DBF_TILE_COLS + 16 * (i & 3));
        } else if (SHARED == 0 && !one_pass) {
            if (stage_a) input_quantise_chunk<true, IN_W>(it, cx, c0, cend);
            else input_quantise_chunk<false, IN_W>(it, cx, c0, cend);
        }
        __syncthreads();
        const bool last_chunk = cend >= ct_end;

        for (int rtl = 0; rtl < it.nrt; rtl += RT_STEP) {
            // ---- stream this wavefront's tiles of (row tile, chunk) -----------------------
            // Slot j is consumed and then refilled in place, so PF-1 loads stay in flight and
            // no register copies are needed; the operand of the next step is read from LDS
            // one step ahead.
            // The operand of a step is read from LDS one step ahead, into the other of two register sets
            // (PF is even, so the sets alternate without copies); its address advances by a constant, the
            // reads of the padded steps at the end run past the operand row into LDS the workgroup owns
            // (their sign operand is zero).  The prefetch cursor advances once per PF steps, in scalar
            // registers; per tile only the lane offset is added.
            static_assert(PF % 2 == 0, "two operand register sets alternate");
            v4i xr[2][NCG];
            v8i xr6[2];  // F4: 32 bf6 values, 24 bytes
            const signed char* xp[NCG];
            auto read6 = [&](int set, const signed char* at) {
                const int* p = reinterpret_cast<const int*>(at);  // (six words, 128 bytes apart)
                xr6[set] = (v8i){p[0], p[32], p[64], p[96], p[128], p[160], 0, 0};
            };
#pragma unroll
            for (int gi = 0; gi < NCG; ++gi) {
                xp[gi] = xq + xrow[gi] + xo_base + w * X_TILE;
                if (F4) read6(0, xp[gi]);
                else if (!RING) xr[0][gi] = *reinterpret_cast<const v4i*>(xp[gi]);
            }
            // (one group = PF tiles; `fresh`: the group's first tile starts the row tile's sums)
            auto group = [&](auto fresh) {
                constexpr bool FRESH = decltype(fresh)::value;
                constexpr int CT_STEP = ROWS ? 1 : WAVES;  // column tiles from one step of a wavefront to the next
                const int g_rt = ROWS ? 4 * p_rt + w : p_rt;
                const int g_ok = (int)(g_rt < it.nrt);
                const int g_ct = ROWS ? c0 + p_i : c0 + w + WAVES * p_i;
                const unsigned g_off = (unsigned)(g_rt * it.n_ct + g_ct) * DBF_TILE_BYTES;
#pragma unroll
                for (int j = 0; j < PF; ++j) {
#pragma unroll
                    for (int gi = 0; gi < NCG; ++gi) {
                        if (F4) read6((j + 1) & 1, xp[gi] + (j + 1) * WAVES * X_TILE);
                        else if (!RING) xr[(j + 1) & 1][gi] = *reinterpret_cast<const v4i*>(xp[gi] + (j + 1) * WAVES * DBF_TILE_COLS);
                    }
                    wait_slot(j);
                    if (F4) {
                        // planes s and 4 + s: the nibble mask 0x1 << s leaves fp4 0.5 / 1 / 2 in both nibbles of a byte; bit 3 of
                        // a nibble alone would be the sign of a zero, so planes 3 and 7 are moved to bit 2 first (2 again)
#pragma unroll
                        for (int s = 0; s < 4; ++s) {
                            const uint32_t msk = s < 3 ? 0x11111111u << s : 0x44444444u;
                            const int sh = s < 3 ? 0 : 1;
                            const v8i a = {(int)((buf[j].x >> sh) & msk), (int)((buf[j].y >> sh) & msk),
                                           (int)((buf[j].z >> sh) & msk), (int)((buf[j].w >> sh) & msk), 0, 0, 0, 0};
                            // (formats: A fp4, B bf6; no scales)
                            accf[s] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, xr6[j & 1], accf[s], 4, 3, 0, 0, 0, 0);
                        }
                    }
#pragma unroll
                    for (int s = 0; s < (F4 ? 0 : 8); ++s) {
                        const uint32_t msk = 0x01010101u << s;
                        v4i a;
                        a.x = (int)(buf[j].x & msk);
                        a.y = (int)(buf[j].y & msk);
                        a.z = (int)(buf[j].z & msk);
                        a.w = (int)(buf[j].w & msk);
#pragma unroll
                        for (int gi = 0; gi < NCG; ++gi)
                            acc[gi][s] = __builtin_amdgcn_mfma_i32_16x16x64_i8(
                                a, RING ? xb[j][gi % XB_N] : xr[j & 1][gi],
                                (FRESH && j == 0) ? (v4i){0, 0, 0, 0} : acc[gi][s], 0, 0, 0);
                    }
                    // (the slot is refilled after the tile's arithmetic.  Refilling it right after the wait, from a copy of the
                    //  tile, was tried: no faster -- 6.18 TB/s either way -- and the compiler then keeps two register homes per
                    //  slot and copies between them at loop ends, while loads are in flight)
                    fetch_at(j, g_off + (unsigned)(j * CT_STEP) * DBF_TILE_BYTES, g_ct + CT_STEP * j,
                             g_ok & (int)(g_ct + CT_STEP * j < cend));
                }
#pragma unroll
                for (int gi = 0; gi < NCG; ++gi) xp[gi] += PF * WAVES * X_TILE;
                const int wrap = (int)(p_i + PF == steps);  // (steps is a multiple of PF)
                p_i = wrap ? 0 : p_i + PF;
                p_rt += wrap;
            };
            int i0 = 0;
            if (SINGLE) {  // (steps >= PF: a chunk is never empty)
                group(std::true_type{});
                i0 = PF;
            }
            for (; i0 < steps; i0 += PF) group(std::false_type{});
            // After the last row tile the ring holds PF placeholder loads that nobody will
            // consume.  They must have landed before the compiler may reuse their registers
            // (it considers them dead from here on): wait, with the slots as operands so that
            // they stay allocated up to this point.  Nothing real is in flight any more, so
            // the wait is short.
            if (rtl + RT_STEP >= it.nrt) retire_ring();
            if (!last_chunk) continue;  // (only with nrt == 1) keep accumulating over chunks

            // ---- combine the wavefronts (integer adds: exact, order independent) -----
            // acc[gi][s][i] of lane (g, c) is row 16*s + 4*g + i, column 16*gi + c.  The two
            // reduction buffers alternate, so one barrier per row tile is enough: a buffer is
            // cleared by its readers one barrier before anybody adds to it again.
            // (ROWS: nothing to combine -- every wavefront has a row tile's whole sums -- but the buffers bring them
            // into the layout of the epilogue: one per wavefront, and a second barrier before they are reused.)
            int* rb = red + (ROWS ? w : (tile_no & 1)) * RB_STRIDE * rcols;
            if (F4) {
                // accf[s][i] of lane (g, c): row 4 g + i of plane s (c < 4) or 4 + s (c in 4..7), digit c & 3, times the
                // operand value of the plane's bit (0.5, 1, 2, 2).  Doubled they are integers; the four digits keep a
                // reduction column each (32 lanes add to 32 different words), and the epilogue puts them together.
                if (c < 8) {
                    int* col = rb + (c & 3) * RB_STRIDE + ((c & 4) ? 64 : 0) + 4 * g;
#pragma unroll
                    for (int s = 0; s < 4; ++s)
#pragma unroll
                        for (int i = 0; i < 4; ++i) atomicAdd(&col[16 * s + i], (int)(accf[s][i] + accf[s][i]));
                }
#pragma unroll
                for (int s = 0; s < 4; ++s) accf[s] = (v4f){0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int gi = 0; gi < (F4 ? 0 : NCG); ++gi) {
                const int col = 16 * gi + c;
                if (col < ncols) {
#pragma unroll
                    for (int s = 0; s < 8; ++s)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            atomicAdd(&rb[col * RB_STRIDE + 4 * g + (16 * s + i)], acc[gi][s][i]);
                }
                if (!SINGLE) {
#pragma unroll
                    for (int s = 0; s < 8; ++s) acc[gi][s] = (v4i){0, 0, 0, 0};
                }
            }
            ++tile_no;
            __syncthreads();
            for (int r4 = 0; r4 < RT_STEP && rtl + r4 < it.nrt; ++r4) {  // the row tiles just finished
                const int rte = rtl + r4;
                if (ROWS) rb = red + r4 * RB_STRIDE * rcols;
                const int row = it.row0 + rte * DBF_TILE_ROWS + rho;
                const float rscale = half_bits_to_float(misc->rscale[rte * DBF_TILE_ROWS + rho]);
                // (threads 0-255; those of wavefronts 4-7 start beyond the batch)
                for (int bi = streams_only ? batch : tid >> 7; bi < batch; bi += 2) {
                    int* ph = &rb[(2 * bi) * RB_STRIDE + rho];  // column-major: [operand column][row of the tile]
                    int vh = ph[0], vl = ph[RB_STRIDE];
                    ph[0] = 0;
                    ph[RB_STRIDE] = 0;
                    if (F4) {
                        // four digit columns, each twice the operand value of the row's plane (1, 2, 4, 4) times the digit
                        // sum: v = d0 + 16 d1 + 256 d2 + 4096 d3; vh * 256 + vl below gives it back
                        const int d2 = ph[2 * RB_STRIDE], d3 = ph[3 * RB_STRIDE];
                        ph[2 * RB_STRIDE] = 0;
                        ph[3 * RB_STRIDE] = 0;
                        const int down = (e_s & 3) < 2 ? (e_s & 3) : 2;
                        const int v = (int)((unsigned)(vh >> down) + ((unsigned)(vl >> down) << 4) + ((unsigned)(d2 >> down) << 8) +
                                            ((unsigned)(d3 >> down) << 12));
                        vl = v & 255;
                        vh = v >> 8;
                    } else if (e_s < 7) {
                        vh >>= e_s;
                        vl >>= e_s;
                    } else {
                        vh = -(vh >> 7);
                        vl = -(vl >> 7);
                    }
                    // (sigma covers the columns this workgroup quantised: its own piece, or, in the one-pass
                    // case, the whole row -- then only the first piece subtracts it)
                    const int sig = (one_pass && ct_first != 0) ? 0 : misc->sigma[bi];
                    // (2 * the sum of the set bits' q may pass 2^31 on the way to a total that fits: modular arithmetic)
                    const int total = (int)(2u * (unsigned)(vh * 256 + vl) - (unsigned)sig);
                    if (n_pieces > 1) {  // a column piece: add the exact integer sum; the last piece to arrive finishes the row
                        __hip_atomic_fetch_add(piece_acc() + (size_t)bi * piece_acc_stride() + rho, total, __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                        continue;
                    }
                    const float val = (float)total * misc->scale[bi] * rscale;
                    if (defer) {
                        // No global store while tiles are in flight: on this chip stores count in the same counter as the
                        // loads, so the ring's next waits -- "at most PF - 1 operations outstanding" -- would wait for the
                        // stores' acknowledgement from memory as well.  (Without the stores in the loop the 512-layer stream
                        // reads 6.9 TB/s instead of 6.1: the whole gap to a bare streaming read.)
                        misc->out[rte * DBF_TILE_ROWS + rho] = val;
                    } else if (stage_a) {
                        // (a workgroup that gave up its wait has read an unfinished t: its outputs say so)
                        if (row < it.rows) y[(size_t)bi * it.rows + row] = misc->gave_up ? HALF_QNAN : float_to_half_bits(val);
                    } else {
                        // agent-scope store: written through to memory, where the A-stage
                        // workgroups of other compute dies read it (padded rows have scale 0)
                        __hip_atomic_store(reinterpret_cast<unsigned*>(it.t) + (size_t)bi * it.t_stride + row,
                                           (F4 && misc->gave_up) ? 0x7FC00000u : __builtin_bit_cast(unsigned, val),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
            if (ROWS) __syncthreads();  // the buffers are clear before the next row tiles' sums arrive
        }
        if (last_chunk) {
            if (defer) {
                // ---- the item's rows, all at once, now that its last tile has been consumed
                __syncthreads();
                for (int idx = tid; idx < it.nrt * DBF_TILE_ROWS; idx += 64 * WAVES) {
                    const int row = it.row0 + idx;
                    const float val = misc->out[idx];
                    if (stage_a) {
                        if (row < it.rows) y[row] = misc->gave_up ? HALF_QNAN : float_to_half_bits(val);
                    } else {
                        __hip_atomic_store(reinterpret_cast<unsigned*>(it.t) + row,
                                           (F4 && misc->gave_up) ? 0x7FC00000u : __builtin_bit_cast(unsigned, val),
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
            if (n_pieces > 1) {
                // ---- column pieces: count this piece in; the last one reads the row tile's sums (and
                // clears them and the counter for the next launch), scales and stores them.  Integer
                // adds are exact, so the result does not depend on the order of arrival.
                asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wavefront's adds have been performed ...
                __syncthreads();                                  // ... and so have the workgroup's
                if (tid == 0) {
                    // low 16 bits: pieces arrived; above: pieces that gave up their wait (their sums are wrong)
                    int* cnt = piece_cnt();
                    const int mine = 1 + (misc->gave_up ? 0x10000 : 0);
                    const int before = __hip_atomic_fetch_add(cnt, mine, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    misc->last = (before & 0xFFFF) == n_pieces - 1;
                    misc->poisoned = ((before + mine) >> 16) != 0;
                    if (misc->last) __hip_atomic_store(cnt, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
                __syncthreads();
                if (misc->last) {
                    const int row = it.row0 + rho;
                    const float rscale = half_bits_to_float(misc->rscale[rho]);
                    for (int bi = tid >> 7; bi < batch; bi += 2) {
                        const int total = __hip_atomic_exchange(piece_acc() + (size_t)bi * piece_acc_stride() + rho, 0,
                                                                __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        const float val = (float)total * misc->scale[bi] * rscale;
                        if (stage_a) {
                            if (row < it.rows) y[(size_t)bi * it.rows + row] = misc->poisoned ? HALF_QNAN : float_to_half_bits(val);
                        } else {
                            __hip_atomic_store(reinterpret_cast<unsigned*>(it.t) + (size_t)bi * it.t_stride + row,
                                               __builtin_bit_cast(unsigned, val), __ATOMIC_RELAXED,
                                               __HIP_MEMORY_SCOPE_AGENT);
                        }
                    }
                }
            }
            break;
        }
        // next chunk (reached only with nrt == 1): restart the tile cursor there
        __syncthreads();  // every wavefront is done reading this chunk's operand
        c0 = cend;
        cend = min(ct_end, c0 + ch_tiles);
        steps = steps_of(cend - c0);
        p_rt = 0;
        p_i = 0;
#pragma unroll
        for (int j = 0; j < PF; ++j) fetch(j);
    }

    // ---- fused launch: a B-stage item publishes its rows of t, an A-stage item counts itself finished.  The
    // counters are per layer (one shared counter for the whole grid would serialise thousands of atomics on one
    // address) and only ever grow; neither add needs its result back.
    if (use_sync) {
        if (!stage_a) {
            // this wavefront's write-through stores of t have been acknowledged by memory ...
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();  // ... and so have those of the whole workgroup
            // (of the pieces of a row tile only the one that stored the result publishes it)
            if (tid == 0 && (n_pieces == 1 || misc->last))
                __hip_atomic_fetch_add(&sync[(size_t)it.layer * DBF_SYNC_STRIDE], (unsigned long long)it.nrt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        } else if (tid == 0 && (n_pieces == 1 || misc->last)) {
            // (of the pieces of a row tile only the one that stored the result counts it)
            __hip_atomic_fetch_add(&sync[(size_t)(n_layers + it.layer) * DBF_SYNC_STRIDE], (unsigned long long)it.nrt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
}

// The input of one stage of every layer of a launch, quantised once: block (layer, batch row) reads the row
// (x times b, or the fp32 middle activations), finds max|u| and writes q = rint(u * 32512 / max|u|) as two
// int8 planes, with the scale and the sum of the q in front (DbfStage::q_in).  The arithmetic is that of the
// items' own prologue (the same functions), so a launch that takes its input from here gives the same bits.
template <bool STAGE_A>
__global__ __launch_bounds__(256) void dbf_quantise_inputs_kernel(const DbfStage* __restrict__ stages,
                                                                 const uint16_t* __restrict__ x_base, int batch) {
    __shared__ Misc misc;
    const DbfStage st = stages[blockIdx.x];
    const int bi = blockIdx.y;
    DbfItem it;
    it.t = st.t + (size_t)bi * st.t_stride;
    it.t_stride = st.t_stride;
    it.in_scale = st.in_scale;
    it.cols = st.cols;
    it.n_ct = st.n_ct;
    const uint16_t* x = x_base + st.x_off * batch;
    // destination: per column tile the 2 * batch planes' 64 bytes one after the other; this row's are 2 bi, 2 bi + 1
    Ctx cx;
    cx.misc = &misc;
    cx.xq = reinterpret_cast<signed char*>(st.q_in + DBF_QIN_HEADER + (size_t)(2 * bi) * DBF_TILE_COLS);
    cx.x = x + (size_t)bi * st.cols;
    cx.chs = DBF_TILE_COLS;
    cx.tstride = 2 * batch * DBF_TILE_COLS;
    cx.tid = threadIdx.x;  cx.lane = threadIdx.x & 63;  cx.w = threadIdx.x >> 6;
    cx.batch = 1;   // this block's row is "batch row 0" of the helpers
    cx.nvec = st.n_ct * 8;
    cx.nvec_x = st.cols >> 3;
    cx.fast = STAGE_A || ((st.cols & 7) == 0 && (reinterpret_cast<uintptr_t>(x) & 15) == 0);
    if (threadIdx.x == 0) misc.sigma[0] = 0;
    __syncthreads();
    if (cx.fast && cx.nvec <= 256 * UNR) {
        // the row fits the registers of the workgroup: read once (plain loads: the middle activations were
        // written by an earlier launch), reduce, quantise from the registers
        v4u r0[UNR], r1[UNR];
#pragma unroll
        for (int j = 0; j < UNR; ++j) {
            const int v = min(256 * j + cx.tid, cx.nvec - 1);
            if (STAGE_A) {
                r0[j] = *reinterpret_cast<const v4u*>(it.t + 8 * (size_t)v);
                r1[j] = *reinterpret_cast<const v4u*>(it.t + 8 * (size_t)v + 4);
            } else {
                const int vx = max(min(v, cx.nvec_x - 1), 0);
                r0[j] = *reinterpret_cast<const v4u*>(cx.x + 8 * (size_t)vx);
                r1[j] = *reinterpret_cast<const v4u*>(it.in_scale + 8 * (size_t)v);
            }
        }
        input_one_pass<STAGE_A, true>(cx, r0, r1);
    } else {
        input_scales<STAGE_A, WIDE>(it, cx);
        input_quantise_chunk<STAGE_A, WIDE, true>(it, cx, 0, st.n_ct);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        reinterpret_cast<float*>(st.q_in)[bi] = misc.scale[0];
        reinterpret_cast<int*>(st.q_in + 64)[bi] = misc.sigma[0];
    }
}

constexpr size_t WIDE_WG_SLACK = 32 * DBF_TILE_COLS;  // extra LDS of an eight-wavefront workgroup (see the launcher)
constexpr int WIDE_WG_MIN_COL_TILES = 32;         // rows shorter than this keep four wavefronts

size_t mfma_smem_bytes(int batch, int ch_tiles, int shared_q, bool f4 = false) {
    const int ncols = 2 * batch;
    // (F4: one operand column per reduction buffer; the operand reads of a row tile's padded steps run past the last
    //  operand row, further than the buffers reach if the row is short: slack for those)
    if (f4) {
        const size_t red = 2 * 4 * (size_t)RB_STRIDE * sizeof(int);  // two buffers of four digit columns
        const int steps = ((ch_tiles + WAVES_F4 - 1) / WAVES_F4 + PF_F4 - 1) / PF_F4 * PF_F4;  // of a wavefront per row tile, padded
        const long over = (long)(WAVES_F4 - 1 + WAVES_F4 * steps + 1 - ch_tiles) * F4_TILE_BYTES;
        const size_t slack = over > (long)red ? (size_t)((over - (long)red + 15) & ~15L) : 0;
        return sizeof(Misc) + (size_t)ch_tiles * F4_TILE_BYTES + red + slack;
    }
    const size_t xq = shared_q >= 2 ? 0 : ((size_t)ncols * (ch_tiles * DBF_TILE_COLS + XQ_PAD) + 15) & ~(size_t)15;
    return sizeof(Misc) + xq + (shared_q == 3 ? 4 : 2) * (size_t)RB_STRIDE * ncols * sizeof(int);
}

}  // namespace

int dbf_mfma_one_pass_cols() { return 256 * UNR * 8; }

int dbf_mfma_chunk_tiles(int batch, int max_cols, int shared_q) {
    const int ncols = 2 * batch;
    // LDS bytes for the quantised operand.  Items that quantise their input themselves keep four workgroups
    // per compute unit; items that copy a shared quantised input (batches of 2 and more) settle for three
    // (52 KiB each, of which the reduction buffers take 1 KiB per operand row) if that lets a whole row stay
    // in LDS, so that an item can take several row tiles.
    int budget = batch > 8 ? 32768 : 28672;
    if (shared_q >= 2) {  // no operand in LDS: the whole row is one "chunk"
        const int all = (dbf_col_tiles(max_cols) + 3) & ~3;
        return all < 4 ? 4 : all;
    }
    if (shared_q) {
        const int roomy = dbf_tune(DBF_TUNE_SHARED_LDS_KB) * 1024 - (int)sizeof(Misc) - 2 * RB_STRIDE * 4 * ncols;
        if (roomy > budget) budget = roomy;
    }
    int ch_tiles = ((budget / ncols - XQ_PAD) / DBF_TILE_COLS) & ~3;
    const int need = (dbf_col_tiles(max_cols) + 3) & ~3;
    if (ch_tiles > need) ch_tiles = need;
    if (ch_tiles < 4) ch_tiles = 4;
    return ch_tiles;
}

// The row-per-wavefront kernels take more than 64 KiB of LDS at the largest batches: the limit has to be raised
// per kernel, once per process.  Called when a launch plan is built -- not at the first launch, which may sit
// inside a stream capture -- and again, for nothing, by the launcher.
hipError_t dbf_mfma_prepare() {
    static const hipError_t raised = [] {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dbf_items_mfma_kernel<1, false, 3, false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dbf_items_mfma_kernel<2, false, 3, false>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e == hipSuccess)
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&dbf_items_mfma_kernel<1, false, 0, true, WAVES_F4, true>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, 80 * 1024);
        if (e != hipSuccess) (void)hipGetLastError();
        return e;
    }();
    return raised;
}

hipError_t dbf_launch_quantise_inputs(const DbfStage* d_stages, int n_layers, int stage_a, const void* x_base,
                                      int batch, hipStream_t stream) {
    if (n_layers <= 0) return hipSuccess;
    const uint16_t* x = static_cast<const uint16_t*>(x_base);
    if (stage_a)
        hipLaunchKernelGGL(dbf_quantise_inputs_kernel<true>, dim3(n_layers, batch), dim3(256), 0, stream, d_stages, x, batch);
    else
        hipLaunchKernelGGL(dbf_quantise_inputs_kernel<false>, dim3(n_layers, batch), dim3(256), 0, stream, d_stages, x, batch);
    return hipGetLastError();
}

hipError_t dbf_launch_items_mfma(const DbfItem* items, int n_items, unsigned long long* sync, int n_layers,
                                 int use_sync, const void* x_base, void* y_base, int batch,
                                 int max_cols, int pieces, int shared_q, int one_pass_rows, int wait_limit_us,
                                 hipStream_t stream) {
    if (n_items <= 0) return hipSuccess;
    const uint16_t* x = static_cast<const uint16_t*>(x_base);
    uint16_t* y = static_cast<uint16_t*>(y_base);
    const int ch_tiles = dbf_mfma_chunk_tiles(batch, max_cols, shared_q);
    const size_t smem = mfma_smem_bytes(batch, ch_tiles, shared_q);
    if (shared_q == 3) {
        const hipError_t raised = dbf_mfma_prepare();  // (done when the plan was built; repeated calls cost nothing)
        if (raised != hipSuccess) return raised;
        if (batch <= 8)
            hipLaunchKernelGGL((dbf_items_mfma_kernel<1, false, 3, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                               n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
        else
            hipLaunchKernelGGL((dbf_items_mfma_kernel<2, false, 3, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                               n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
        return hipGetLastError();
    }
    // column pieces (small batches only)
    if (shared_q == 2 && batch <= 8)
        hipLaunchKernelGGL((dbf_items_mfma_kernel<1, false, 2, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                           n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    else if (shared_q == 2)
        hipLaunchKernelGGL((dbf_items_mfma_kernel<2, false, 2, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                           n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    else if (shared_q && batch <= 8)
        hipLaunchKernelGGL((dbf_items_mfma_kernel<1, false, 1, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                           n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    else if (shared_q)
        hipLaunchKernelGGL((dbf_items_mfma_kernel<2, false, 1, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                           n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    else if (pieces)
        hipLaunchKernelGGL((dbf_items_mfma_kernel<1, true, 0, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                           n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    else if (batch == 1 && one_pass_rows && dbf_col_tiles(max_cols) <= F4_MAX_COL_TILES &&
             dbf_col_tiles(max_cols) >= WIDE_WG_MIN_COL_TILES && n_items <= dbf_tune(DBF_TUNE_FP4_MAX_ITEMS)) {
        // (every row of the launch takes the one-pass prologue, and the launch does not fill the chip: the fp4 x bf6 form.
        //  One layer alone, back to back, int8 form with four / eight wavefronts / this form: 4096 x 4096 at k = 4096 11.6 /
        //  11.0 / 10.8 us, k = 2048 10.5 / 10.1 / 9.8, 2048 columns 9.3 / 9.0 / 8.7, 4096 -> 11008 11.2 / 11.2 / 10.9; 1024 columns
        //  8.4 / 8.4 / 8.6, hence the column limit.  Streams lose with it -- 512 layers of 4096 x 4096 5.9 against 6.1 TB/s, 256 layers
        //  5.5 / 5.9, 1024 x 4096 at 1 bit 3.3 / 4.3 -- its operand rows fill LDS at two workgroups per compute unit, and
        //  its prologue is the longer one)
        const hipError_t raised = dbf_mfma_prepare();  // (done when the plan was built; repeated calls cost nothing)
        if (raised != hipSuccess) return raised;
        const int tiles4 = (dbf_col_tiles(max_cols) + 3) & ~3;
        hipLaunchKernelGGL((dbf_items_mfma_kernel<1, false, 0, true, WAVES_F4, true>), dim3(n_items), dim3(64 * WAVES_F4),
                           mfma_smem_bytes(1, tiles4, 0, true), stream, items, sync, n_layers, use_sync, x, y, batch, tiles4,
                           wait_limit_us);
    } else if (batch <= 8 && ch_tiles >= dbf_col_tiles(max_cols) && n_items <= dbf_tune(DBF_TUNE_WIDE_WG_MAX_ITEMS) &&
             dbf_col_tiles(max_cols) >= WIDE_WG_MIN_COL_TILES)
        // (few items of long rows: eight wavefronts each.  One layer alone, back to back: 4096 x 4096 11.6 -> 11.1 us,
        //  2048 columns 9.4 -> 9.1, 512 columns 8.3 -> 9.1: the wider workgroup costs 0.4 us to start.  A wavefront's
        //  operand reads for the padded steps at the end of a row tile run up to 31 column tiles past the operand
        //  row: LDS the workgroup owns)
        hipLaunchKernelGGL((dbf_items_mfma_kernel<1, false, 0, true, 8>), dim3(n_items), dim3(512), smem + WIDE_WG_SLACK,
                           stream, items, sync, n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    else if (batch <= 8 && ch_tiles >= dbf_col_tiles(max_cols))
        hipLaunchKernelGGL((dbf_items_mfma_kernel<1, false, 0, true>), dim3(n_items), dim3(256), smem, stream, items, sync,
                           n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    else if (batch <= 8)
        hipLaunchKernelGGL((dbf_items_mfma_kernel<1, false, 0, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                           n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    else
        hipLaunchKernelGGL((dbf_items_mfma_kernel<2, false, 0, false>), dim3(n_items), dim3(256), smem, stream, items, sync,
                           n_layers, use_sync, x, y, batch, ch_tiles, wait_limit_us);
    return hipGetLastError();
}
