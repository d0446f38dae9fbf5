// One ADMM update of the factorisation (paper, section 3.2, the three-line update after the SVID
// definition), with the two matrices that stay constant while B and W are fixed formed by the caller:
//
//     Minv = (B^T B + rho I)^-1  (q x q),   C = B^T W  (q x r)
//
//     R  = C + rho (a . S . m^T - U)           dbf_admm_rhs_kernel     (A = a . S . m^T never exists densely:
//                                                                       S is read from the packed tile layout)
//     Z  = Minv^T R + U   (= W_hat + U)        dbf_admm_gemm_kernel    fp32 matrix cores, U added in the epilogue
//     (S', a', m') = SVID(Z)                   dbf_svid (dbf_svid.hip)
//     U' = Z - a' . S' . m'^T  (= U + W_hat - A')   dbf_admm_dual_kernel
//
// The contraction is q x q x r in fp32 (34 GFLOP at q = 2048, r = 4096) and dominates; the elementwise
// kernels and the projection are bandwidth bound.  The paper gives no kernel design for this step.
#include "dbf_kernels.h"

#include <cmath>

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));

// ---------------------------------------------------------------------------------------------
// Elementwise kernels.  One workgroup per 128 x 64 tile of the sign matrix; thread t takes the four
// columns 4 (t % 16) .. + 3 of rows 16 s + t / 16, s = 0 .. 7.  Their eight sign quadruples are the
// eight bits of the four bytes of ONE 32-bit word of the tile (byte 256 g + 16 r + j, bit s = sign of
// row 16 s + r, column 16 g + j), and a wavefront touches four rows of 256 contiguous bytes per pass.
// ---------------------------------------------------------------------------------------------
struct TileThread {
    int row0, col, word;  // first row (s = 0), first column, word index in the tile
};
__device__ inline TileThread tile_thread(int t) {
    const int rr = t >> 4, cq = t & 15;
    TileThread x;
    x.row0 = blockIdx.y * DBF_TILE_ROWS + rr;
    x.col = blockIdx.x * DBF_TILE_COLS + 4 * cq;
    x.word = 64 * (cq >> 2) + 4 * rr + (cq & 3);
    return x;
}

// MODE 0: out = C + rho (a_i m_j s_ij - U)     (in1 = C, in2 = U)
// MODE 1: out = Z - a_i m_j s_ij               (in1 = Z; out may be any buffer but Z)
template <int MODE>
__global__ __launch_bounds__(256) void dbf_admm_elementwise_kernel(const float* __restrict__ in1,
                                                                  const float* __restrict__ in2, float rho,
                                                                  const float* __restrict__ a,
                                                                  const float* __restrict__ m,
                                                                  const uint8_t* __restrict__ bits, int rows, int cols,
                                                                  int n_ct, int vec_ok, float* __restrict__ out) {
    const TileThread x = tile_thread(threadIdx.x);
    if (x.col >= cols) return;
    const unsigned w =
        reinterpret_cast<const unsigned*>(bits + ((size_t)blockIdx.y * n_ct + blockIdx.x) * DBF_TILE_BYTES)[x.word];
    const bool vec = vec_ok && x.col + 4 <= cols;
    float mj[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) mj[e] = x.col + e < cols ? m[x.col + e] : 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int row = x.row0 + 16 * s;
        if (row >= rows) break;
        const float ai = a[row];
        const size_t at = (size_t)row * cols + x.col;
        float v1[4], v2[4] = {0.f, 0.f, 0.f, 0.f}, res[4];
        if (vec) {
            const v4f p = *reinterpret_cast<const v4f*>(in1 + at);
            v1[0] = p.x;  v1[1] = p.y;  v1[2] = p.z;  v1[3] = p.w;
            if (MODE == 0) {
                const v4f u = *reinterpret_cast<const v4f*>(in2 + at);
                v2[0] = u.x;  v2[1] = u.y;  v2[2] = u.z;  v2[3] = u.w;
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                v1[e] = x.col + e < cols ? in1[at + e] : 0.f;
                if (MODE == 0) v2[e] = x.col + e < cols ? in2[at + e] : 0.f;
            }
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float am = ai * mj[e];
            const float A = ((w >> (8 * e + s)) & 1u) ? am : -am;
            res[e] = MODE == 0 ? v1[e] + rho * (A - v2[e]) : v1[e] - A;
        }
        if (vec) {
            *reinterpret_cast<v4f*>(out + at) = (v4f){res[0], res[1], res[2], res[3]};
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (x.col + e < cols) out[at + e] = res[e];
        }
    }
}

// ---------------------------------------------------------------------------------------------
// out = alpha (P^T Q) . rs . cs^T + add + diag I on the fp32 matrix cores:
//     out[i][j] = alpha * rs[i] * cs[j] * sum_k P[k][i] Q[k][j] + add[i][j] + (i == j ? diag : 0).
// Both operands are read by rows of k ("k major"), which is how v_mfma_f32_32x32x2_f32 wants them
// (lane l supplies A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32]), so tiles go from memory
// to LDS without a transpose.  Workgroup = 128 x 128 outputs, 4 wavefronts of 64 x 64 (2 x 2 blocks of
// 32 x 32: 64 accumulator registers); 16 values of k per step, double buffered in LDS, the next step's
// tiles in registers while the current one is multiplied; one barrier per step (32 matrix instructions
// of 64 cycles per wavefront).  Rows of the LDS tiles are padded by 32 floats so that the two halves of
// a wavefront (k and k + 1) read different banks.
// Workgroups are renumbered so that a compute die (linear id modulo 8) works on neighbouring column
// blocks: the Q tiles it needs stay in its own L2.
//
// An operand may also be a packed sign matrix S (rows = the operand's output index, columns = k) in the
// 128 x 64 tile layout, scaled per k: P[k][i] = kscale[k] * S[i][k] (template arguments PS / QS).  The 16 x 128
// operand slice of a step is 256 bytes of one tile (the step's 16 columns are one byte group g, byte
// 16 r + j of it holds in bit s the sign of row 16 s + r, column 16 g + j): 64 threads read one word each and
// write its 4 x 8 values to LDS.  Padding bits of the tiles are zero bits, i.e. -1, not zero: columns beyond K
// get a zero scale here, rows beyond M are never stored.  This is how the fixed factor of the ADMM update
// stays in its packed form: B^T B and B^T W are formed from the sign bits directly.
// ---------------------------------------------------------------------------------------------
constexpr int GT = 128;         // outputs per workgroup side
#ifndef DBF_ADMM_GK
#define DBF_ADMM_GK 16
#endif
constexpr int GK = DBF_ADMM_GK; // values of k per step
constexpr int GLD = GT + 32;    // LDS row length in floats
static_assert(GK == 16, "a step of a sign operand is one 16-column byte group of a tile");

struct GemmArgs {
    const float* P;        // dense [K][M], leading dimension ldp           (PS == false)
    const float* Q;        // dense [K][N], leading dimension ldq           (QS == false)
    const uint8_t* Pbits;  // packed signs, rows = i (M of them), cols = k  (PS == true); first tile of row i = 0
    const uint8_t* Qbits;  // the same for j                                (QS == true)
    const float* kscale;   // [K] scale per k of the sign operands
    const float* add;      // [M][N] with leading dimension lda, or NULL
    const float* rs;       // [M] or NULL
    const float* cs;       // [N] or NULL
    float* out;            // [M][N], leading dimension ldo (may be `add`: every element is read before it is written)
    size_t ldp, ldq, lda, ldo;
    float alpha, diag;
    int M, N, K;
    int bits_nct;          // column tiles of the sign matrices
    int vec_p, vec_q;      // rows of P / Q can be read in 16-byte pieces
    int upper;             // symmetric output: workgroups whose block lies wholly below the diagonal do nothing
    int ktri;              // both operands are lower triangular in (k, output index), i.e. zero for k < index: the
                           // summation starts at the first k that can contribute to the block
};

__device__ inline v4f load_row4(const float* base, size_t ld, int k, int K, int c, int C, int vec) {
    if (k >= K || c >= C) return (v4f){0.f, 0.f, 0.f, 0.f};
    const float* p = base + (size_t)k * ld + c;
    if (vec && c + 4 <= C) return *reinterpret_cast<const v4f*>(p);
    v4f r = {0.f, 0.f, 0.f, 0.f};
    r.x = p[0];
    if (c + 1 < C) r.y = p[1];
    if (c + 2 < C) r.z = p[2];
    if (c + 3 < C) r.w = p[3];
    return r;
}

template <bool PS, bool QS>
__global__ __launch_bounds__(256) void dbf_admm_gemm_kernel(const GemmArgs g) {
    __shared__ __align__(16) float As[2][GK][GLD];
    __shared__ __align__(16) float Bs[2][GK][GLD];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned n_wg = gridDim.x * gridDim.y, lin = blockIdx.x + gridDim.x * blockIdx.y;
    const unsigned die = lin & 7, slot = lin >> 3, per = n_wg >> 3, extra = n_wg & 7;
    const unsigned vid = die * per + (die < extra ? die : extra) + slot;
    const int i0 = (int)(vid % gridDim.x) * GT, j0 = (int)(vid / gridDim.x) * GT;
    if (g.upper && i0 >= j0 + GT) return;
    const int wi = (w & 1) * 64, wj = (w >> 1) * 64;  // this wavefront's 64 x 64 corner in the tile
    const int l32 = lane & 31, h = lane >> 5;

    // staging role, dense operand: GK / 8 16-byte pieces of a tile per thread: rows k = tid / 32 (+ 8, ...),
    // columns 4 (tid % 32).  Sign operand: threads 0..63 take word tid of the step's 256 bytes (wavefront 0 for P,
    // wavefront 1 for Q, so that the two do not queue behind each other).
    constexpr int NP = GK / 8;
    const int sk = tid >> 5, sc = 4 * (tid & 31);
    v4f ra[NP], rb[NP];
    unsigned sa = 0, sb = 0;
    float ka[4] = {0.f, 0.f, 0.f, 0.f}, kb[4] = {0.f, 0.f, 0.f, 0.f};
    const int st = tid & 63;                       // word of the step
    const int s_r = st >> 2, s_j = 4 * (st & 3);   // row within the 16-row group, first of its 4 columns
    const uint8_t* p_tiles = PS ? g.Pbits + (size_t)(i0 / DBF_TILE_ROWS) * g.bits_nct * DBF_TILE_BYTES : nullptr;
    const uint8_t* q_tiles = QS ? g.Qbits + (size_t)(j0 / DBF_TILE_ROWS) * g.bits_nct * DBF_TILE_BYTES : nullptr;
    auto fetch_signs = [&](const uint8_t* tiles, int k0, unsigned& word, float (&ks)[4]) {
        // (k0 is a multiple of 16: tile k0 / 64, byte group (k0 % 64) / 16)
        const int kk = min(k0, (g.bits_nct * DBF_TILE_COLS) - GK);
        word = reinterpret_cast<const unsigned*>(tiles + (size_t)(kk >> 6) * DBF_TILE_BYTES + 256 * ((kk >> 4) & 3))[st];
#pragma unroll
        for (int e = 0; e < 4; ++e) ks[e] = (k0 + s_j + e < g.K) ? g.kscale[k0 + s_j + e] : 0.f;
    };
    auto fetch = [&](int k0) {
        if (PS) {
            if (w == 0) fetch_signs(p_tiles, k0, sa, ka);
        } else {
#pragma unroll
            for (int e = 0; e < NP; ++e) ra[e] = load_row4(g.P, g.ldp, k0 + sk + 8 * e, g.K, i0 + sc, g.M, g.vec_p);
        }
        if (QS) {
            if (w == 1) fetch_signs(q_tiles, k0, sb, kb);
        } else {
#pragma unroll
            for (int e = 0; e < NP; ++e) rb[e] = load_row4(g.Q, g.ldq, k0 + sk + 8 * e, g.K, j0 + sc, g.N, g.vec_q);
        }
    };
    auto stage_signs = [&](float (*dst)[GLD], unsigned word, const float (&ks)[4]) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
#pragma unroll
            for (int s = 0; s < 8; ++s) dst[s_j + e][16 * s + s_r] = ((word >> (8 * e + s)) & 1u) ? ks[e] : -ks[e];
    };
    auto stage = [&](int buf) {
        if (PS) {
            if (w == 0) stage_signs(As[buf], sa, ka);
        } else {
#pragma unroll
            for (int e = 0; e < NP; ++e) *reinterpret_cast<v4f*>(&As[buf][sk + 8 * e][sc]) = ra[e];
        }
        if (QS) {
            if (w == 1) stage_signs(Bs[buf], sb, kb);
        } else {
#pragma unroll
            for (int e = 0; e < NP; ++e) *reinterpret_cast<v4f*>(&Bs[buf][sk + 8 * e][sc]) = rb[e];
        }
    };

    v16f acc[2][2];
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0.f;

    // (lower triangular operands: P[k][i] = 0 for k < i and Q[k][j] = 0 for k < j, so k starts at the larger of
    //  the block's first row and first column -- a multiple of the step)
    const int k_first = g.ktri ? max(i0, j0) : 0;
    const int steps = (g.K - k_first + GK - 1) / GK;
    // (the operand values of k pair kk + 1 are read from LDS before the matrix instructions of pair kk are
    // issued, into the other of two register sets: the LDS latency then hides behind 256 cycles of matrix work)
    auto multiply = [&](int buf) {
        float fa[2][2], fb[2][2];
        auto read_pair = [&](int kk, int set) {
            fa[set][0] = As[buf][2 * kk + h][wi + l32];
            fa[set][1] = As[buf][2 * kk + h][wi + 32 + l32];
            fb[set][0] = Bs[buf][2 * kk + h][wj + l32];
            fb[set][1] = Bs[buf][2 * kk + h][wj + 32 + l32];
        };
        read_pair(0, 0);
#pragma unroll
        for (int kk = 0; kk < GK / 2; ++kk) {
            const int set = kk & 1;
            if (kk + 1 < GK / 2) read_pair(kk + 1, set ^ 1);
            __builtin_amdgcn_sched_barrier(0);  // (keeps the reads above the matrix instructions)
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[set][0], fb[set][0], acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[set][0], fb[set][1], acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[set][1], fb[set][0], acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[set][1], fb[set][1], acc[1][1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    // A workgroup whose dense tiles lie wholly inside both operands (and whose rows can be read in 16-byte pieces)
    // takes a loop without a single branch: guarded loads put a wait for memory between the request and the
    // matrix instructions of every step.  The last step requests its own tiles once more instead of none.
    const bool inside = !PS && !QS && g.vec_p && g.vec_q && i0 + GT <= g.M && j0 + GT <= g.N && (g.K - k_first) % GK == 0;
    if (inside) {
        const float* pa = g.P + (size_t)(k_first + sk) * g.ldp + i0 + sc;
        const float* pb = g.Q + (size_t)(k_first + sk) * g.ldq + j0 + sc;
        auto fetch_inside = [&](int k0) {
#pragma unroll
            for (int e = 0; e < NP; ++e) {
                ra[e] = *reinterpret_cast<const v4f*>(pa + (size_t)(k0 + 8 * e) * g.ldp);
                rb[e] = *reinterpret_cast<const v4f*>(pb + (size_t)(k0 + 8 * e) * g.ldq);
            }
        };
        fetch_inside(0);
        stage(0);
        __syncthreads();
        for (int s = 0; s < steps; ++s) {
            fetch_inside(min(s + 1, steps - 1) * GK);
            multiply(s & 1);
            stage((s & 1) ^ 1);
            __syncthreads();
        }
    } else {
        fetch(k_first);
        stage(0);
        __syncthreads();
        for (int s = 0; s < steps; ++s) {
            if (s + 1 < steps) fetch(k_first + (s + 1) * GK);
            multiply(s & 1);
            if (s + 1 < steps) stage((s & 1) ^ 1);
            __syncthreads();
        }
    }

    // epilogue: register v of lane l of a 32 x 32 block is row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj) {
            const int col = j0 + wj + 32 * bj + l32;
            if (col >= g.N) continue;
            const float csj = g.cs ? g.cs[col] * g.alpha : g.alpha;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wi + 32 * bi + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row < g.M) {
                    float val = acc[bi][bj][v] * csj;
                    if (g.rs) val *= g.rs[row];
                    if (g.add) val += g.add[(size_t)row * g.lda + col];
                    if (row == col) val += g.diag;
                    g.out[(size_t)row * g.ldo + col] = val;
                }
            }
        }
}

// A dense call: out (M x N, leading dimension ldo) = P^T Q, P [K][M] with leading dimension ldp, Q [K][N] with ldq.
inline GemmArgs dense_gemm(const float* P, size_t ldp, const float* Q, size_t ldq, float* out, size_t ldo, int M, int N,
                           int K) {
    GemmArgs g;
    g.P = P;  g.Q = Q;  g.Pbits = nullptr;  g.Qbits = nullptr;  g.kscale = nullptr;
    g.add = nullptr;  g.rs = nullptr;  g.cs = nullptr;  g.out = out;
    g.ldp = ldp;  g.ldq = ldq;  g.lda = 0;  g.ldo = ldo;
    g.alpha = 1.f;  g.diag = 0.f;
    g.M = M;  g.N = N;  g.K = K;
    g.bits_nct = 0;
    auto vec = [](const float* p, size_t ld) { return (p && (ld & 3) == 0 && (reinterpret_cast<uintptr_t>(p) & 15) == 0) ? 1 : 0; };
    g.vec_p = vec(P, ldp);
    g.vec_q = vec(Q, ldq);
    g.upper = 0;
    g.ktri = 0;
    return g;
}
template <bool PS, bool QS>
inline void launch_gemm(const GemmArgs& g, hipStream_t st) {
    if (g.M < 1 || g.N < 1 || g.K < 1) return;
    hipLaunchKernelGGL((dbf_admm_gemm_kernel<PS, QS>), dim3((g.M + GT - 1) / GT, (g.N + GT - 1) / GT), dim3(256), 0, st, g);
}

// ---------------------------------------------------------------------------------------------
// Cholesky factorisation G = R^T R (R upper triangular) of the symmetric positive definite
// G = B^T B + rho I and its inverse, blocked by 128 (the contraction kernel's tile):
//   for every block column:  factor the 128 x 128 diagonal block and invert its factor (one workgroup,
//   in LDS: below);  R[jb, j>jb] = R_jj^-T G[jb, j>jb]  and  G[i>jb, j>jb] -= R[jb, i]^T R[jb, j]  are calls of
//   the contraction kernel above (both operands k major as they lie in memory, no transposes).
//   Y = R^-T (lower triangular) from the identity, right-looking:  Y[i, :] = R_ii^-T Y[i, :], then
//   Y[i' > i, :] -= R[i, i']^T Y[i, :];   G^-1 = Y^T Y, one more contraction (upper blocks, then mirrored).
// Only the upper triangle of G is ever read.
// ---------------------------------------------------------------------------------------------
constexpr int NB = GT;  // block size of the factorisation

// One workgroup: the w x w diagonal block at (j0, j0) of G (leading dimension ld) is replaced by its upper
// Cholesky factor (zeros below the diagonal); tinv (NB x NB, row major) receives the inverse of that factor,
// the identity on the padded part.  *fail is raised if a pivot is not positive (G not positive definite).
//
// The factorisation keeps the block in registers: the 256 threads form a 16 x 16 grid, thread (ti, tj) owns
// the elements (16 a + ti, 16 b + tj), a, b < 8.  A step = one pivot row c: its owners put the row into LDS
// (two buffers alternate: one barrier per step), everybody reads the pivot and the 8 + 8 row entries that
// meet its own rows and columns, scales them by 1 / sqrt(pivot), and subtracts their products from its
// elements of the rows below c.  The row index 16 ca + cr is walked with ca unrolled, so every register index
// is a constant.  Only the upper triangle is meaningful; what accumulates below it is never used.
__global__ __launch_bounds__(256) void dbf_chol_diag_kernel(float* __restrict__ G, size_t ld, int j0, int w,
                                                          float* __restrict__ tinv, int* __restrict__ fail) {
    constexpr int LDA = NB + 4;  // (rows 16 bytes aligned; neighbouring rows four banks apart)
    __shared__ __align__(16) float A[NB][LDA];
    __shared__ __align__(16) float T[NB][LDA];
    __shared__ __align__(16) float tmp[8][16][16];
    __shared__ float rowbuf[2][NB];
    const int tid = threadIdx.x, ti = tid >> 4, tj = tid & 15;
    float reg[8][8];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int i = 16 * a + ti, j = 16 * b + tj;
            float v = (i == j) ? 1.f : 0.f;                  // padding: identity
            if (i < w && j < w && j >= i) v = G[(size_t)(j0 + i) * ld + j0 + j];
            reg[a][b] = v;
        }
    int bad = 0;
#pragma unroll
    for (int ca = 0; ca < 8; ++ca) {
        for (int cr = 0; cr < 16; ++cr) {
            const int c = 16 * ca + cr;
            float* rb = rowbuf[c & 1];
            if (ti == cr) {
#pragma unroll
                for (int b = ca; b < 8; ++b) rb[16 * b + tj] = reg[ca][b];
            }
            __syncthreads();
            const float piv = rb[c];
            float inv = 0.f;
            if (piv > 0.f) inv = 1.f / sqrtf(piv); else bad = 1;
            float ri[8], rj[8];
#pragma unroll
            for (int a = ca; a < 8; ++a) ri[a] = rb[16 * a + ti] * inv;
#pragma unroll
            for (int b = ca; b < 8; ++b) rj[b] = rb[16 * b + tj] * inv;
            if (ti == cr) {                                   // the pivot row itself becomes row c of the factor
#pragma unroll
                for (int b = ca; b < 8; ++b) reg[ca][b] = rj[b];
            }
#pragma unroll
            for (int a = ca; a < 8; ++a) {
                const bool below = a > ca || ti > cr;          // rows after c
#pragma unroll
                for (int b = ca; b < 8; ++b)
                    if (below) reg[a][b] -= ri[a] * rj[b];
            }
        }
    }
    if (bad && tid == 0) atomicAdd(fail, 1);                  // (every thread saw the same pivots)
    // the factor to LDS (for the inverse) and to memory, zeros below the diagonal
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b = 0; b < 8; ++b) {
            const int i = 16 * a + ti, j = 16 * b + tj;
            const float v = j >= i ? reg[a][b] : 0.f;
            A[i][j] = v;
            T[i][j] = 0.f;
            if (i < w && j < w) G[(size_t)(j0 + i) * ld + j0 + j] = v;
        }
    __syncthreads();
    // Inverse of the upper triangular factor by 16 x 16 blocks.  The eight diagonal blocks first: thread (I, cc),
    // 128 of them, solves R_II x = e_cc from the last row upwards with x in registers (entries beyond cc come out
    // as zeros by themselves, so every index is a constant).
    if (tid < NB) {
        const int I = tid >> 4, cc = tid & 15;
        float x[16];
#pragma unroll
        for (int i = 15; i >= 0; --i) {
            float acc = (i == cc) ? 1.f : 0.f;
#pragma unroll
            for (int l = i + 1; l < 16; ++l) acc -= A[16 * I + i][16 * I + l] * x[l];
            const float di = A[16 * I + i][16 * I + i];
            x[i] = di != 0.f ? acc / di : 0.f;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) T[16 * I + i][16 * I + cc] = x[i];
    }
    __syncthreads();
    // Then block diagonal by block diagonal, d = J - I = 1 .. 7 (the blocks of one diagonal are independent):
    //     T_IJ = -T_II * (sum over I < K <= J of R_IK T_KJ),
    // thread (r, cc) takes element (r, cc) of every block of the diagonal; the inner sum goes through LDS.
    {
        const int r = ti, cc = tj;
        for (int d = 1; d < 8; ++d) {
            for (int I = 0; I + d < 8; ++I) {
                const int J = I + d;
                float acc = 0.f;
                for (int K = I + 1; K <= J; ++K) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc += A[16 * I + r][16 * K + e] * T[16 * K + e][16 * J + cc];
                }
                tmp[I][r][cc] = acc;
            }
            __syncthreads();
            for (int I = 0; I + d < 8; ++I) {
                const int J = I + d;
                float acc = 0.f;
#pragma unroll
                for (int e = 0; e < 16; ++e) acc += T[16 * I + r][16 * I + e] * tmp[I][e][cc];
                T[16 * I + r][16 * J + cc] = -acc;
            }
            __syncthreads();
        }
    }
    for (int e = tid; e < NB * NB; e += 256) tinv[e] = T[e / NB][e % NB];
}

// Y = identity (q x q).
__global__ __launch_bounds__(256) void dbf_chol_identity_kernel(float* __restrict__ Y, int q) {
    const int row = blockIdx.y;
    const int col = blockIdx.x * 256 + threadIdx.x;
    if (col < q) Y[(size_t)row * q + col] = row == col ? 1.f : 0.f;
}

// M[j][i] = M[i][j] for i < j: the lower triangle of a symmetric matrix whose upper blocks were computed.
// One workgroup per 32 x 32 block on or above the diagonal, through LDS so that both sides are coalesced.
__global__ __launch_bounds__(256) void dbf_chol_mirror_kernel(float* __restrict__ M, int q) {
    __shared__ float t[32][33];
    const int bi = blockIdx.y, bj = blockIdx.x;
    if (bi > bj) return;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int rr = ty; rr < 32; rr += 8) {
        const int i = 32 * bi + rr, j = 32 * bj + tx;
        t[rr][tx] = (i < q && j < q) ? M[(size_t)i * q + j] : 0.f;
    }
    __syncthreads();
    for (int rr = ty; rr < 32; rr += 8) {
        const int j = 32 * bj + rr, i = 32 * bi + tx;   // writes M[j][i] = t[i - 32 bi][j - 32 bj]
        if (i < q && j < q && i < j) M[(size_t)j * q + i] = t[tx][rr];
    }
}

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
struct AdmmWorkspace {
    size_t R, Z, svid, total;
};
inline AdmmWorkspace admm_workspace(int q, int r) {
    AdmmWorkspace w;
    size_t off = 0;
    w.R = off;     off = up256(off + 4 * (size_t)q * r);
    w.Z = off;     off = up256(off + 4 * (size_t)q * r);
    w.svid = off;  off = up256(off + dbf_svid_workspace_bytes(q, r));
    w.total = off;
    return w;
}

}  // namespace

extern "C" size_t dbf_admm_workspace_bytes(int q, int r) {
    if (q < 1 || r < 1 || q > DBF_MAX_DIM || r > DBF_MAX_DIM) return 0;
    return admm_workspace(q, r).total;
}

extern "C" int dbf_admm_step(const void* Minv_dev, const void* C_dev, int q, int r, float rho, int svid_iters,
                             void* a_dev, void* m_dev, void* bits_dev, void* U_dev, void* workspace_dev,
                             size_t workspace_bytes, void* hip_stream) {
    if (!Minv_dev || !C_dev || !a_dev || !m_dev || !bits_dev || !U_dev) return DBF_EINVAL;
    if (q < 1 || r < 1 || q > DBF_MAX_DIM || r > DBF_MAX_DIM || svid_iters < 1) return DBF_EINVAL;
    if (!(rho > 0.f) || !std::isfinite(rho)) return DBF_EINVAL;
    const void* ptrs[6] = {Minv_dev, C_dev, a_dev, m_dev, bits_dev, U_dev};
    for (const void* p : ptrs)
        if (reinterpret_cast<uintptr_t>(p) & 3) return DBF_EINVAL;
    const AdmmWorkspace w = admm_workspace(q, r);
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) || workspace_bytes < w.total)
        return DBF_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    uint8_t* base = static_cast<uint8_t*>(workspace_dev);
    float* R = reinterpret_cast<float*>(base + w.R);
    float* Z = reinterpret_cast<float*>(base + w.Z);
    float* U = static_cast<float*>(U_dev);
    const float* C = static_cast<const float*>(C_dev);
    const int n_rt = dbf_row_tiles(q), n_ct = dbf_col_tiles(r);
    auto aligned16 = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
    const int vec_r = ((r & 3) == 0 && aligned16(C) && aligned16(U)) ? 1 : 0;  // (R and Z are 256-byte aligned)

    hipLaunchKernelGGL(dbf_admm_elementwise_kernel<0>, dim3(n_ct, n_rt), dim3(256), 0, st, C, U, rho,
                       static_cast<const float*>(a_dev), static_cast<const float*>(m_dev),
                       static_cast<const uint8_t*>(bits_dev), q, r, n_ct, vec_r, R);
    GemmArgs g = dense_gemm(static_cast<const float*>(Minv_dev), q, R, r, Z, r, q, r, q);
    g.add = U;
    g.lda = r;
    launch_gemm<false, false>(g, st);
    if (hipGetLastError() != hipSuccess) return DBF_EHIP;
    const int rc = dbf_svid(Z, q, r, svid_iters, a_dev, m_dev, bits_dev, base + w.svid, workspace_bytes - w.svid, st);
    if (rc != DBF_OK) return rc;
    hipLaunchKernelGGL(dbf_admm_elementwise_kernel<1>, dim3(n_ct, n_rt), dim3(256), 0, st, Z, nullptr, 0.f,
                       static_cast<const float*>(a_dev), static_cast<const float*>(m_dev),
                       static_cast<const uint8_t*>(bits_dev), q, r, n_ct, vec_r, U);
    if (hipGetLastError() != hipSuccess) return DBF_EHIP;
    return DBF_OK;
}

// ---- forming the constant matrices of the update on the device ---------------------------------
namespace {
struct PrepWorkspace {
    size_t Y, tinv, fail, total;
    int nblk;
};
inline PrepWorkspace prep_workspace(int q) {
    PrepWorkspace w;
    w.nblk = (q + NB - 1) / NB;
    size_t off = 0;
    w.Y = off;     off = up256(off + 4 * (size_t)q * q);
    w.tinv = off;  off = up256(off + 4 * (size_t)w.nblk * NB * NB);
    w.fail = off;  off = up256(off + 256);
    w.total = off;
    return w;
}
__global__ void dbf_admm_clear_flag_kernel(int* flag) { *flag = 0; }
}  // namespace

extern "C" size_t dbf_admm_prepare_workspace_bytes(int p, int q, int r) {
    if (p < 1 || q < 1 || r < 1 || p > DBF_MAX_DIM || q > DBF_MAX_DIM || r > DBF_MAX_DIM) return 0;
    return prep_workspace(q).total;
}

extern "C" int dbf_admm_prepare(const void* bits_dev, const void* m2_dev, const void* b_dev, const void* W_dev, int p,
                                int q, int r, float rho, void* Minv_dev, void* C_dev, void* workspace_dev,
                                size_t workspace_bytes, int* not_positive_definite_dev, void* hip_stream) {
    if (!bits_dev || !m2_dev || !b_dev || !W_dev || !Minv_dev || !C_dev) return DBF_EINVAL;
    if (p < 1 || q < 1 || r < 1 || p > DBF_MAX_DIM || q > DBF_MAX_DIM || r > DBF_MAX_DIM) return DBF_EINVAL;
    if (!(rho > 0.f) || !std::isfinite(rho)) return DBF_EINVAL;
    const void* ptrs[7] = {bits_dev, m2_dev, b_dev, W_dev, Minv_dev, C_dev, not_positive_definite_dev};
    for (const void* ptr : ptrs)
        if (reinterpret_cast<uintptr_t>(ptr) & 3) return DBF_EINVAL;
    const PrepWorkspace w = prep_workspace(q);
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) || workspace_bytes < w.total)
        return DBF_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    uint8_t* base = static_cast<uint8_t*>(workspace_dev);
    float* Y = reinterpret_cast<float*>(base + w.Y);
    float* tinv = reinterpret_cast<float*>(base + w.tinv);
    int* fail = not_positive_definite_dev ? not_positive_definite_dev : reinterpret_cast<int*>(base + w.fail);
    float* G = static_cast<float*>(Minv_dev);  // G, then its factor, live in the output until the last contraction
    const uint8_t* bits = static_cast<const uint8_t*>(bits_dev);
    const float* m2 = static_cast<const float*>(m2_dev);
    const float* b = static_cast<const float*>(b_dev);
    const int n_ct = dbf_col_tiles(p);

    hipLaunchKernelGGL(dbf_admm_clear_flag_kernel, dim3(1), dim3(1), 0, st, fail);
    // G = B^T B + rho I with B[l][j] = b_l S[j][l] m2_j: both operands are the sign tiles, scaled by b per summation
    // index, m2 by output row and column in the epilogue.  Upper blocks only.
    {
        GemmArgs g = dense_gemm(nullptr, 0, nullptr, 0, G, q, q, q, p);
        g.Pbits = bits;  g.Qbits = bits;  g.kscale = b;  g.bits_nct = n_ct;
        g.rs = m2;  g.cs = m2;  g.diag = rho;  g.upper = 1;
        launch_gemm<true, true>(g, st);
    }
    // C = B^T W: the sign tiles against the dense W
    {
        GemmArgs g = dense_gemm(nullptr, 0, static_cast<const float*>(W_dev), r, static_cast<float*>(C_dev), r, q, r, p);
        g.Pbits = bits;  g.kscale = b;  g.bits_nct = n_ct;
        g.rs = m2;
        launch_gemm<true, false>(g, st);
    }
    // G = R^T R
    for (int jb = 0; jb < w.nblk; ++jb) {
        const int j0 = jb * NB, wb = q - j0 < NB ? q - j0 : NB, rest = q - j0 - wb;
        float* tj = tinv + (size_t)jb * NB * NB;
        hipLaunchKernelGGL(dbf_chol_diag_kernel, dim3(1), dim3(256), 0, st, G, (size_t)q, j0, wb, tj, fail);
        if (rest > 0) {
            // panel: R[j0 + i][j0 + wb + j] = sum_k tinv[k][i] G[j0 + k][j0 + wb + j]   (in place: a workgroup has
            // read all of its columns before it writes them)
            float* panel = G + (size_t)j0 * q + j0 + wb;
            GemmArgs g1 = dense_gemm(tj, NB, panel, q, panel, q, wb, rest, wb);
            launch_gemm<false, false>(g1, st);
            // trailing update: G[i][j] -= sum_k R[j0 + k][i] R[j0 + k][j], upper blocks
            float* trail = G + (size_t)(j0 + wb) * q + j0 + wb;
            GemmArgs g2 = dense_gemm(panel, q, panel, q, trail, q, rest, rest, wb);
            g2.alpha = -1.f;  g2.add = trail;  g2.lda = q;  g2.upper = 1;
            launch_gemm<false, false>(g2, st);
        }
    }
    // Y = R^-T (lower triangular), right-looking so that every call has many workgroups: Y starts as the identity;
    // block row ib is finished by Y[ib, :] = R_ii^-T Y[ib, :], then every later block row loses its share
    // Y[i', :] -= R[ib, i']^T Y[ib, :].  Only the columns up to the block's own are non-zero.
    hipLaunchKernelGGL(dbf_chol_identity_kernel, dim3((q + 255) / 256, q), dim3(256), 0, st, Y, q);
    for (int ib = 0; ib < w.nblk; ++ib) {
        const int i0 = ib * NB, wb = q - i0 < NB ? q - i0 : NB, rest = q - i0 - wb, ncol = i0 + wb;
        const float* ti = tinv + (size_t)ib * NB * NB;
        float* yrow = Y + (size_t)i0 * q;
        // (in place: a workgroup has read all of its columns before it writes them)
        GemmArgs g1 = dense_gemm(ti, NB, yrow, q, yrow, q, wb, ncol, wb);
        launch_gemm<false, false>(g1, st);
        if (rest > 0) {
            float* ynext = Y + (size_t)(i0 + wb) * q;
            GemmArgs g2 = dense_gemm(G + (size_t)i0 * q + i0 + wb, q, yrow, q, ynext, q, rest, ncol, wb);
            g2.alpha = -1.f;  g2.add = ynext;  g2.lda = q;
            launch_gemm<false, false>(g2, st);
        }
    }
    // G^-1 = Y^T Y (overwrites the factor): upper blocks, the sums starting where both operands can be non-zero,
    // then the mirror image
    {
        GemmArgs g = dense_gemm(Y, q, Y, q, G, q, q, q, q);
        g.upper = 1;  g.ktri = 1;
        launch_gemm<false, false>(g, st);
        hipLaunchKernelGGL(dbf_chol_mirror_kernel, dim3((q + 31) / 32, (q + 31) / 32), dim3(256), 0, st, G, q);
    }
    if (hipGetLastError() != hipSuccess) return DBF_EHIP;
    return DBF_OK;
}
