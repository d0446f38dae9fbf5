// Prefill: the layer product for T tokens as two fp16 matrix-core contractions.
//
//   stage 1:  mid = ((X . b) B^T) . m      (T x k,     contraction over n_in)
//   stage 2:  Y   = (mid A^T) . a          (T x n_out, contraction over k)
//
// (forward-pass expression of the paper, section 3; the paper times batch 1 only, so this
// kernel design is not taken from it).  At hundreds of tokens the sign products really are
// dense contractions, so they run on v_mfma_f32_16x16x32_f16 with fp32 accumulation:
//
//   * The sign matrix is the A operand.  The tile layout already gives lane (r, g) sixteen
//     columns of row 16*s + r in bit s of its sixteen bytes, which is exactly "row r,
//     k-group g" of the instruction.  One shift and one bit-field insert turn a loaded word
//     into a register of two fp16 values -1/+1 (bytes 0 and 2, or 1 and 3, of the word), so a
//     sign costs one vector-ALU operation and is then used for every token block.
//   * That pairing fixes the order of the eight k-slots of a lane as columns (0,2,1,3,4,6,5,7)
//     of its 8-column block; the X tile is written to LDS in the same order, so the B operand
//     is one 16-byte LDS read.
//   * The inserted sign bit is set where the stored bit is set (+1), i.e. the operand is the
//     NEGATED sign matrix; the epilogue multiplies by minus the row scale.
//   * b is folded into the X tile when it is staged (fp32 product rounded once to fp16),
//     m and a are applied to the fp32 accumulators in the epilogues, mid is stored as fp16.
//
// Work split: a workgroup of 8 wavefronts computes 512 rows x 64 tokens.  Wavefronts w and w + 4
// share the 128-row tile w of the block and sit on the same SIMD: each expands only four of the
// eight bit planes of the sign tile (64 of its rows; 4 row groups x 4 token blocks = 16
// accumulator tiles), so that the vector-ALU sign expansion of one overlaps the matrix
// instructions of the other -- a single wavefront issues in order and would do one after the
// other.  All eight share the 64-token X tile in LDS (double buffered, one barrier per 64
// columns); the first four stage it.
#include "dbf_kernels.h"

namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));

constexpr int GM_TOKENS = 64;            // tokens per workgroup
constexpr int GM_ROWTILES = 4;           // 128-row tiles per workgroup (one per pair of wavefronts)
constexpr int GM_THREADS = 512;
constexpr int XROW_BYTES = 64 * 2 + 16;  // one token's 64 fp16 columns + padding (LDS banks)
constexpr int GM_DEPTH = 4;              // 64-column steps requested ahead of the one being computed

struct GemmArgs {
    const uint8_t* bits;        // tiled sign matrix of the stage: n_rt x n_ct tiles
    const uint16_t* col_scale;  // fp16 [n_ct*64] (b, zero padded) or NULL
    const uint16_t* row_scale;  // fp16 [n_rt*128] (m or a, zero padded)
    const uint16_t* X;          // fp16 [T][ldx]
    uint16_t* out;              // fp16 [T][ldo]
    int n_rt, n_ct;
    int T, ldx, ldo;
    int k_valid;                // valid columns of X (reads beyond are replaced by zero)
    int n_valid;                // valid output rows (columns of `out`) to store
    int x_vec_ok;               // X rows can be read with 16-byte loads
};

// (mask & a) | (~mask & b) as ONE v_bfi_b32.  Written as an instruction because with two constant
// operands the compiler prefers an AND and an OR; all three operands are kept in registers.
__device__ inline unsigned bfi(unsigned mask, unsigned a, unsigned b) {
    unsigned d;
    asm("v_bfi_b32 %0, %1, %2, %3" : "=v"(d) : "v"(mask), "v"(a), "v"(b));
    return d;
}
__device__ inline float h2f(uint16_t h) { return (float)__builtin_bit_cast(_Float16, h); }
__device__ inline unsigned pack2(float lo, float hi) {
    h2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(unsigned, v);
}

// Sixteen consecutive fp16 columns of one token, loaded from global memory.
struct XRegs {
    v4u lo, hi;      // columns 0..7 and 8..15 of the thread's 16-column block
    v4u slo, shi;    // stage 1: the same columns of the scale vector b (requested together with X,
                     // so that staging never waits for them)
};

template <bool HAS_COLSCALE>
__device__ inline XRegs load_x(const GemmArgs& a, int token, int col0) {
    XRegs r;
    r.lo = (v4u){0, 0, 0, 0};
    r.hi = (v4u){0, 0, 0, 0};
    r.slo = (v4u){0, 0, 0, 0};
    r.shi = (v4u){0, 0, 0, 0};
    if (HAS_COLSCALE && col0 < a.k_valid) {  // b is zero padded up to a multiple of 64 columns
        const v4u* sp = reinterpret_cast<const v4u*>(a.col_scale + col0);
        r.slo = sp[0];
        r.shi = sp[1];
    }
    if (token >= a.T) return r;
    const uint16_t* row = a.X + (size_t)token * a.ldx;
    if (a.x_vec_ok && col0 + 16 <= a.k_valid) {
        const v4u* p = reinterpret_cast<const v4u*>(row + col0);
        r.lo = p[0];
        r.hi = p[1];
    } else if (col0 < a.k_valid) {
        unsigned w[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int c0 = col0 + 2 * i, c1 = c0 + 1;
            const unsigned v0 = c0 < a.k_valid ? row[c0] : 0u;
            const unsigned v1 = c1 < a.k_valid ? row[c1] : 0u;
            w[i] = v0 | (v1 << 16);
        }
        r.lo = (v4u){w[0], w[1], w[2], w[3]};
        r.hi = (v4u){w[4], w[5], w[6], w[7]};
    }
    return r;
}

// Scales the 16 columns (stage 1) and writes them to LDS with every group of four columns in
// the order (0, 2, 1, 3), the order of the k-slots of the expanded sign operand.
template <bool HAS_COLSCALE>
__device__ inline void store_x(const GemmArgs& a, const XRegs& r, unsigned char* dst, int col0) {
    const unsigned in[8] = {r.lo.x, r.lo.y, r.lo.z, r.lo.w, r.hi.x, r.hi.y, r.hi.z, r.hi.w};
    unsigned out[8];
    if (HAS_COLSCALE) {
        // (beyond the matrix both X and the scale registers are zero)
        const v4u s0 = r.slo, s1 = r.shi;
        const unsigned sc[8] = {s0.x, s0.y, s0.z, s0.w, s1.x, s1.y, s1.z, s1.w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {  // four columns 4q .. 4q+3
            const float u0 = h2f(in[2 * q] & 0xFFFF) * h2f(sc[2 * q] & 0xFFFF);
            const float u1 = h2f(in[2 * q] >> 16) * h2f(sc[2 * q] >> 16);
            const float u2 = h2f(in[2 * q + 1] & 0xFFFF) * h2f(sc[2 * q + 1] & 0xFFFF);
            const float u3 = h2f(in[2 * q + 1] >> 16) * h2f(sc[2 * q + 1] >> 16);
            out[2 * q] = pack2(u0, u2);
            out[2 * q + 1] = pack2(u1, u3);
        }
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const unsigned a01 = in[2 * q], a23 = in[2 * q + 1];
            out[2 * q] = (a01 & 0xFFFFu) | (a23 << 16);
            out[2 * q + 1] = (a01 >> 16) | (a23 & 0xFFFF0000u);
        }
    }
    v4u* d = reinterpret_cast<v4u*>(dst);
    d[0] = (v4u){out[0], out[1], out[2], out[3]};
    d[1] = (v4u){out[4], out[5], out[6], out[7]};
}

template <bool HAS_COLSCALE>
__global__ __launch_bounds__(GM_THREADS) void dbf_gemm_stage_kernel(const GemmArgs a) {
    __shared__ __align__(16) unsigned char xs[2][GM_TOKENS * XROW_BYTES];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int g = lane >> 4, c = lane & 15;
    const int token0 = blockIdx.y * GM_TOKENS;
    const int rt = blockIdx.x * GM_ROWTILES + (w & 3);  // this wavefront's row tile
    const int sh = w >> 2;                              // ... and its half of the bit planes
    const bool stager = w < 4;                          // stages X into LDS
    const bool active = rt < a.n_rt;              // wavefronts beyond the matrix only help staging X
    const v4u* tiles = reinterpret_cast<const v4u*>(a.bits) + (size_t)(active ? rt : 0) * a.n_ct * 64 + lane;

    // staging role: thread -> (token, 16-column block)
    const int s_tok = tid >> 2, s_col = (tid & 3) * 16;
    unsigned char* s_dst0 = xs[0] + s_tok * XROW_BYTES + s_col * 2;
    unsigned char* s_dst1 = xs[1] + s_tok * XROW_BYTES + s_col * 2;

    v4f acc[4][4];
#pragma unroll
    for (int s = 0; s < 4; ++s)
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) acc[s][tb] = (v4f){0.f, 0.f, 0.f, 0.f};

    // constants of the sign expansion, held in registers (see bfi)
    unsigned sign_mask = 0x80008000u, one_one = 0x3C003C00u;
    asm volatile("" : "+v"(sign_mask), "+v"(one_one));

    // Software pipeline over the 64-column steps.  With one wavefront per SIMD nothing else hides
    // memory latency, so the X columns and the sign tile of step kt + GM_DEPTH are requested
    // while step kt is computed; the loop is unrolled GM_DEPTH times so that every in-flight
    // register has a fixed name.  Steps beyond the matrix (the count is rounded up to a
    // multiple of GM_DEPTH) stage zeros for X and therefore add nothing.
    XRegs xr[GM_DEPTH];
    v4u bq[GM_DEPTH];
    const int last_ct = a.n_ct - 1;
#pragma unroll
    for (int j = 0; j < GM_DEPTH; ++j) {
        if (stager) xr[j] = load_x<HAS_COLSCALE>(a, token0 + s_tok, j * 64 + s_col);
        bq[j] = tiles[(size_t)min(j, last_ct) * 64];
    }
    if (stager) store_x<HAS_COLSCALE>(a, xr[0], s_dst0, s_col);
    __syncthreads();

    for (int kt0 = 0; kt0 < a.n_ct; kt0 += GM_DEPTH) {
#pragma unroll
        for (int j = 0; j < GM_DEPTH; ++j) {
            const int kt = kt0 + j;
            // xr[j] held step kt, which was staged one step ago: reuse it for step kt + GM_DEPTH
            // Stage step kt + 1 first (its columns were requested GM_DEPTH - 1 steps ago; the
            // buffer it goes to was last read in step kt - 1, which the barrier has closed), so
            // that the staging wavefronts reach the barrier at the end of this step together
            // with the others instead of keeping them waiting.
            if (stager) {
                store_x<HAS_COLSCALE>(a, xr[(j + 1) % GM_DEPTH], (j & 1) ? s_dst0 : s_dst1, (kt + 1) * 64 + s_col);
                xr[j] = load_x<HAS_COLSCALE>(a, token0 + s_tok, (kt + GM_DEPTH) * 64 + s_col);
            }
            const unsigned char* xb = xs[j & 1] + c * XROW_BYTES + 32 * g;
            // (wavefronts beyond the matrix compute on row tile 0 and discard the result: a
            // branch around the matrix instructions would make the compiler shuttle all 128
            // accumulators between the two register files on every iteration)
            // this wavefront's bit planes 4*sh .. 4*sh+3, moved down to planes 0..3
            const unsigned wd[4] = {bq[j].x >> (4 * sh), bq[j].y >> (4 * sh), bq[j].z >> (4 * sh),
                                    bq[j].w >> (4 * sh)};
            // Eight (half, plane) rounds of four matrix instructions each.  A wavefront issues in
            // order, so the expansion of the NEXT round's operand (four shift + insert pairs) is
            // written, and pinned by scheduling barriers, between the matrix instructions of the
            // current round: one pair after each of them keeps the matrix pipe fed.
            auto expand = [&](int r, int part) -> unsigned {
                // round r = 4*h + s; parts x, y, z, w hold the fp16 pairs whose sign bits are bits
                // (s, 16+s) resp. (8+s, 24+s) of the two words of half h
                const int h = r >> 2, s = r & 3;
                const unsigned word = wd[2 * h + (part >> 1)];
                return bfi(sign_mask, word << ((part & 1) ? 7 - s : 15 - s), one_one);
            };
            v8h xf[2][4];
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int tb = 0; tb < 4; ++tb)
                    xf[h][tb] = *reinterpret_cast<const v8h*>(xb + tb * 16 * XROW_BYTES + 16 * h);
            v4u e_next;
            e_next.x = expand(0, 0);
            e_next.y = expand(0, 1);
            e_next.z = expand(0, 2);
            e_next.w = expand(0, 3);
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const int h = r >> 2, s = r & 3;
                const v8h av = __builtin_bit_cast(v8h, e_next);
                const int rn = r < 7 ? r + 1 : 7;  // (the last round re-expands itself: unused)
                acc[s][0] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, xf[h][0], acc[s][0], 0, 0, 0);
                const unsigned n0 = expand(rn, 0);
                acc[s][1] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, xf[h][1], acc[s][1], 0, 0, 0);
                const unsigned n1 = expand(rn, 1);
                acc[s][2] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, xf[h][2], acc[s][2], 0, 0, 0);
                const unsigned n2 = expand(rn, 2);
                acc[s][3] = __builtin_amdgcn_mfma_f32_16x16x32_f16(av, xf[h][3], acc[s][3], 0, 0, 0);
                const unsigned n3 = expand(rn, 3);
                e_next = (v4u){n0, n1, n2, n3};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one matrix instruction
                    __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);  // two vector-ALU instructions
                }
            }
            bq[j] = tiles[(size_t)min(kt + GM_DEPTH, last_ct) * 64];
            __syncthreads();
        }
    }

    // ---- epilogue: acc[s][tb][i] of lane (g, c) is row 16*s + 4*g + i, token 16*tb + c --------
    if (!active) return;
    const bool vec_ok = (a.ldo & 3) == 0 && (reinterpret_cast<uintptr_t>(a.out) & 7) == 0;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
        const int n0 = rt * DBF_TILE_ROWS + 16 * (4 * sh + s) + 4 * g;
        float rs[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) rs[i] = -h2f(a.row_scale[n0 + i]);  // operand was the negated signs
#pragma unroll
        for (int tb = 0; tb < 4; ++tb) {
            const int token = token0 + 16 * tb + c;
            if (token >= a.T) continue;
            uint16_t* dst = a.out + (size_t)token * a.ldo + n0;
            const float v0 = acc[s][tb].x * rs[0], v1 = acc[s][tb].y * rs[1];
            const float v2 = acc[s][tb].z * rs[2], v3 = acc[s][tb].w * rs[3];
            if (vec_ok && n0 + 4 <= a.n_valid) {
                *reinterpret_cast<uint2*>(dst) = make_uint2(pack2(v0, v1), pack2(v2, v3));
            } else {
                const float v[4] = {v0, v1, v2, v3};
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (n0 + i < a.n_valid) dst[i] = __builtin_bit_cast(uint16_t, (_Float16)v[i]);
            }
        }
    }
}

inline size_t mid_stride(const dbf_layer* L) { return (size_t)dbf_row_tiles(L->k) * DBF_TILE_ROWS; }

}  // namespace

size_t dbf_gemm_f16_workspace_bytes(const dbf_layer* L, int T) {
    return ((size_t)T * mid_stride(L) * 2 + 255) & ~(size_t)255;
}

// Launches the two fp16 stages on `stream`.  Arguments are validated by the caller (dbf_gemm);
// `workspace_dev` holds at least dbf_gemm_f16_workspace_bytes(L, T) bytes.
hipError_t dbf_gemm_f16_launch(const dbf_layer* L, const void* X_dev, void* Y_dev, int T, void* workspace_dev,
                               hipStream_t stream) {
    const int ks = (int)mid_stride(L);
    const unsigned tok_blocks = (unsigned)((T + GM_TOKENS - 1) / GM_TOKENS);

    GemmArgs s1;
    s1.bits = L->dB;  s1.col_scale = L->db;  s1.row_scale = L->dm;
    s1.X = static_cast<const uint16_t*>(X_dev);
    s1.out = static_cast<uint16_t*>(workspace_dev);
    s1.n_rt = dbf_row_tiles(L->k);  s1.n_ct = dbf_col_tiles(L->n_in);
    s1.T = T;  s1.ldx = L->n_in;  s1.ldo = ks;
    s1.k_valid = L->n_in;
    s1.n_valid = ks;  // padded rows have m = 0 and are written as zeros: stage 2 reads them
    s1.x_vec_ok = ((L->n_in & 7) == 0 && (reinterpret_cast<uintptr_t>(X_dev) & 15) == 0) ? 1 : 0;
    hipLaunchKernelGGL(dbf_gemm_stage_kernel<true>,
                       dim3((s1.n_rt + GM_ROWTILES - 1) / GM_ROWTILES, tok_blocks), dim3(GM_THREADS), 0, stream, s1);
    if (hipGetLastError() != hipSuccess) return hipErrorUnknown;

    GemmArgs s2;
    s2.bits = L->dA;  s2.col_scale = nullptr;  s2.row_scale = L->da;
    s2.X = static_cast<const uint16_t*>(workspace_dev);
    s2.out = static_cast<uint16_t*>(Y_dev);
    s2.n_rt = dbf_row_tiles(L->n_out);  s2.n_ct = dbf_col_tiles(L->k);
    s2.T = T;  s2.ldx = ks;  s2.ldo = L->n_out;
    s2.k_valid = s2.n_ct * DBF_TILE_COLS;  // <= ks, zero beyond k
    s2.n_valid = L->n_out;
    s2.x_vec_ok = 1;
    hipLaunchKernelGGL(dbf_gemm_stage_kernel<false>,
                       dim3((s2.n_rt + GM_ROWTILES - 1) / GM_ROWTILES, tok_blocks), dim3(GM_THREADS), 0, stream, s2);
    return hipGetLastError();
}
