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
// Z = Mt^T R + U on the fp32 matrix cores: Z[i][j] = sum_k Mt[k][i] R[k][j] + U[i][j].
// Both operands are read by rows of k ("k major"), which is how v_mfma_f32_32x32x2_f32 wants them
// (lane l supplies A[i = l % 32][k = l / 32] and B[k = l / 32][j = l % 32]), so tiles go from memory
// to LDS without a transpose.  Workgroup = 128 x 128 outputs, 4 wavefronts of 64 x 64 (2 x 2 blocks of
// 32 x 32: 64 accumulator registers); 16 values of k per step, double buffered in LDS, the next step's
// tiles in registers while the current one is multiplied; one barrier per step (32 matrix instructions
// of 64 cycles per wavefront).  Rows of the LDS tiles are padded by 32 floats so that the two halves of
// a wavefront (k and k + 1) read different banks.
// Workgroups are renumbered so that a compute die (linear id modulo 8) works on neighbouring column
// blocks: the R tiles it needs stay in its own L2.
// ---------------------------------------------------------------------------------------------
constexpr int GT = 128;         // outputs per workgroup side
#ifndef DBF_ADMM_GK
#define DBF_ADMM_GK 16
#endif
constexpr int GK = DBF_ADMM_GK; // values of k per step
constexpr int GLD = GT + 32;    // LDS row length in floats

struct GemmArgs {
    const float* Mt;   // [K][M] row major
    const float* R;    // [K][N] row major
    const float* U;    // [M][N]
    float* Z;          // [M][N]
    int M, N, K;
    int vec_m, vec_n;  // rows of Mt / R can be read in 16-byte pieces
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

__global__ __launch_bounds__(256) void dbf_admm_gemm_kernel(const GemmArgs g) {
    __shared__ __align__(16) float As[2][GK][GLD];
    __shared__ __align__(16) float Bs[2][GK][GLD];

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned n_wg = gridDim.x * gridDim.y, lin = blockIdx.x + gridDim.x * blockIdx.y;
    const unsigned die = lin & 7, slot = lin >> 3, per = n_wg >> 3, extra = n_wg & 7;
    const unsigned vid = die * per + (die < extra ? die : extra) + slot;
    const int i0 = (int)(vid % gridDim.x) * GT, j0 = (int)(vid / gridDim.x) * GT;
    const int wi = (w & 1) * 64, wj = (w >> 1) * 64;  // this wavefront's 64 x 64 corner in the tile
    const int l32 = lane & 31, h = lane >> 5;

    // staging role: GK / 8 16-byte pieces of each tile per thread: rows k = tid / 32 (+ 8, ...), columns 4 (tid % 32)
    constexpr int NP = GK / 8;
    const int sk = tid >> 5, sc = 4 * (tid & 31);
    v4f ra[NP], rb[NP];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int e = 0; e < NP; ++e) {
            ra[e] = load_row4(g.Mt, (size_t)g.M, k0 + sk + 8 * e, g.K, i0 + sc, g.M, g.vec_m);
            rb[e] = load_row4(g.R, (size_t)g.N, k0 + sk + 8 * e, g.K, j0 + sc, g.N, g.vec_n);
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int e = 0; e < NP; ++e) {
            *reinterpret_cast<v4f*>(&As[buf][sk + 8 * e][sc]) = ra[e];
            *reinterpret_cast<v4f*>(&Bs[buf][sk + 8 * e][sc]) = rb[e];
        }
    };

    v16f acc[2][2];
#pragma unroll
    for (int bi = 0; bi < 2; ++bi)
#pragma unroll
        for (int bj = 0; bj < 2; ++bj)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[bi][bj][v] = 0.f;

    const int steps = (g.K + GK - 1) / GK;
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
    // A workgroup whose tiles lie wholly inside both operands (and whose rows can be read in 16-byte pieces)
    // takes a loop without a single branch: guarded loads put a wait for memory between the request and the
    // matrix instructions of every step.  The last step requests its own tiles once more instead of none.
    const bool inside = g.vec_m && g.vec_n && i0 + GT <= g.M && j0 + GT <= g.N && g.K % GK == 0;
    if (inside) {
        const float* pa = g.Mt + (size_t)sk * g.M + i0 + sc;
        const float* pb = g.R + (size_t)sk * g.N + j0 + sc;
        auto fetch_inside = [&](int k0) {
#pragma unroll
            for (int e = 0; e < NP; ++e) {
                ra[e] = *reinterpret_cast<const v4f*>(pa + (size_t)(k0 + 8 * e) * g.M);
                rb[e] = *reinterpret_cast<const v4f*>(pb + (size_t)(k0 + 8 * e) * g.N);
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
        fetch(0);
        stage(0);
        __syncthreads();
        for (int s = 0; s < steps; ++s) {
            if (s + 1 < steps) fetch((s + 1) * GK);
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
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = i0 + wi + 32 * bi + 8 * (v >> 2) + 4 * h + (v & 3);
                if (row < g.M) {
                    const size_t at = (size_t)row * g.N + col;
                    g.Z[at] = acc[bi][bj][v] + g.U[at];
                }
            }
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
    GemmArgs g;
    g.Mt = static_cast<const float*>(Minv_dev);
    g.R = R;
    g.U = U;
    g.Z = Z;
    g.M = q;
    g.N = r;
    g.K = q;
    g.vec_m = ((q & 3) == 0 && aligned16(Minv_dev)) ? 1 : 0;
    g.vec_n = (r & 3) == 0 ? 1 : 0;
    hipLaunchKernelGGL(dbf_admm_gemm_kernel, dim3((q + GT - 1) / GT, (r + GT - 1) / GT), dim3(256), 0, st, g);
    if (hipGetLastError() != hipSuccess) return DBF_EHIP;
    const int rc = dbf_svid(Z, q, r, svid_iters, a_dev, m_dev, bits_dev, base + w.svid, workspace_bytes - w.svid, st);
    if (rc != DBF_OK) return rc;
    hipLaunchKernelGGL(dbf_admm_elementwise_kernel<1>, dim3(n_ct, n_rt), dim3(256), 0, st, Z, nullptr, 0.f,
                       static_cast<const float*>(a_dev), static_cast<const float*>(m_dev),
                       static_cast<const uint8_t*>(bits_dev), q, r, n_ct, vec_r, U);
    if (hipGetLastError() != hipSuccess) return DBF_EHIP;
    return DBF_OK;
}
