// SVID projection (paper, section 3.2): SVID(Z) = a . Sign(Z) . m^T, where a m^T is the rank-one
// decomposition of |Z| obtained by power iteration.  It is the projection step of the ADMM iteration
// that computes the factorisation; here it produces the sign matrix directly in the packed device
// tile layout of this library (what a layer stores), and the two scale vectors in fp32.
//
// Readings of what the paper leaves open (the same as the CPU oracle's): Sign(0) = +1; the iteration
// starts from the constant unit vector and runs `iters` rounds of
//     u <- |Z| v / ||.||,   v <- |Z|^T u,   sigma <- ||v||,   v <- v / sigma;      a = sigma u,  m = v.
//
// Everything is bound by reading Z (fp32, rows x cols, row major).  A round needs u = |Z| v before any of
// v' = |Z|^T u -- but only row by row: the term of row i in v' needs u_i alone, and u_i needs row i alone.  So
// ONE pass over Z does a whole round (dbf_svid_round_kernel): a workgroup of 16 wavefronts holds a batch of whole
// rows in registers, forms their dots with v, and adds the rows, weighted by those dots, into its partial column
// sums; a second, small launch sums the partial sums over the workgroups.  Rows too long for that (more than
// 24576 columns) or not readable in 16-byte pieces, and matrices of fewer than 24 Mi entries (where it is slower),
// take two passes per round (row dots, column dots) and a reduce launch.  In both forms the normalisations are not passes of their own.  The iterate is kept unnormalised (u_raw = |Z| v, v_raw = |Z|^T u_raw; the length of u
// cancels in v / ||v||), the column reduction leaves the squared length of v_raw as one partial sum per
// workgroup, and the next row pass scales by 1 / ||v_raw|| on the fly; the last kernel forms
// m = v_raw / ||v_raw|| and a = sigma u = u_raw ||v_raw|| / ||u_raw||^2.  All reductions have a fixed
// order, so the result does not depend on scheduling:
//   row dots     one wavefront per row, 16-byte loads, butterfly reduction;
//   column dots  workgroup = 256 columns x 64 rows (4 row lanes x 16 rows, combined in LDS in lane
//                order), partial sums per 64-row chunk, then summed over the chunks in a fixed order;
//   norms        partial sums of squares per 64 columns (v) or per thread stride (u), combined in a fixed tree;
//   signs        one workgroup per 128 x 64 tile, a thread per four bytes of the tile.
#include "dbf_kernels.h"
#include "dbf_wave.h"

namespace {

typedef float v4f __attribute__((ext_vector_type(4)));

constexpr int COL_CHUNK_ROWS = 64;   // rows per partial sum of the column pass
constexpr int COL_BLOCK = 256;       // columns per workgroup of the column pass
constexpr int ROUND_THREADS = 1024;  // workgroup of the one-pass round
// Matrices below this many entries take the two-pass round: a workgroup of the one-pass round then holds too few
// rows to keep its loads ahead of its barriers.  Measured, 8 rounds, two passes / one pass in ms: 4096 x 4096 0.254 /
// 0.299, 2048 x 4096 0.183 / 0.221, 6144 x 4096 0.361 / 0.336, 11008 x 4096 0.587 / 0.452, 4096 x 11008 0.507 / 0.410,
// 16384 x 4096 0.866 / 0.578, 8192 x 8192 0.933 / 0.551.
constexpr size_t ROUND_MIN_ENTRIES = (size_t)24 << 20;

__device__ inline float wave_sum_f(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Sum of n partial sums in a fixed order (lane-strided, then butterfly); every lane gets the result.
__device__ inline float wave_total(const float* __restrict__ part, int n, int lane) {
    float s = 0.f;
    for (int i = lane; i < n; i += 64) s += part[i];
    return wave_sum_f(s);
}

// u_raw[i] = (sum_j |Z[i][j]| v_raw[j]) / ||v_raw||, with ||v_raw||^2 = sum of ss_part[0 .. n_ss).
// FIRST: the start vector, v = 1 / sqrt(cols) everywhere (v_raw and ss_part are not read).
template <bool FIRST>
__global__ __launch_bounds__(256) void dbf_svid_row_dots_kernel(const float* __restrict__ Z, int rows, int cols,
                                                               const float* __restrict__ v,
                                                               const float* __restrict__ ss_part, int n_ss,
                                                               float* __restrict__ u, int vec_ok) {
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const float* z = Z + (size_t)row * cols;
    float s = 0.f;
    if (vec_ok) {
        for (int c = 4 * lane; c < cols; c += 256) {
            const v4f a = *reinterpret_cast<const v4f*>(z + c);
            if (FIRST) {
                s += (fabsf(a.x) + fabsf(a.y)) + (fabsf(a.z) + fabsf(a.w));
            } else {
                const v4f b = *reinterpret_cast<const v4f*>(v + c);
                s += fabsf(a.x) * b.x + fabsf(a.y) * b.y + fabsf(a.z) * b.z + fabsf(a.w) * b.w;
            }
        }
    } else {
        for (int c = lane; c < cols; c += 64) s += FIRST ? fabsf(z[c]) : fabsf(z[c]) * v[c];
    }
    s = wave_sum_f(s);
    float inv;
    if (FIRST) {
        inv = 1.0f / sqrtf((float)cols);
    } else {
        const float nrm = sqrtf(wave_total(ss_part, n_ss, lane));
        inv = nrm > 0.f ? 1.0f / nrm : 0.f;
    }
    if (lane == 0) u[row] = s * inv;
}

// One round in one pass.  Workgroup = 1024 threads = 16 wavefronts, one per compute unit (512-thread workgroups,
// two or three per compute unit, were slower); it takes `rows_per_wg` consecutive rows, RB at a time.  Thread t
// holds, of every row of the batch, the CPL float4s at columns 4 t + 4096 k (k < CPL), so a wavefront's load of a
// row segment is 1 KiB contiguous.  Per batch: the next batch's loads are issued first (register double buffer:
// the barrier below puts all 16 wavefronts in step, so nothing else hides the latency), then every wavefront
// forms its part of the RB row dots (register-to-register reduction), leaves it in LDS, and after ONE barrier
// (two LDS buffers alternate) every thread sums the 16 parts in wavefront order, scales by 1 / ||v_raw|| -> u_raw
// of the RB rows (threads 0 .. RB-1 store them), and adds |z| u_raw of its columns into its CPL float4
// accumulators.  At the end the accumulators are the workgroup's partial column sums: partial[workgroup][column].
// FIRST: v = 1 / sqrt(cols) everywhere, v_raw is not read.  All sums have a fixed order.
template <int CPL, bool FIRST>
__global__ __launch_bounds__(ROUND_THREADS) void dbf_svid_round_kernel(const float* __restrict__ Z, int rows, int cols,
                                                              const float* __restrict__ v,
                                                              const float* __restrict__ ss_part, int n_ss,
                                                              float* __restrict__ u, float* __restrict__ partial,
                                                              int rows_per_wg) {
    constexpr int RB = CPL == 1 ? 8 : CPL == 2 ? 4 : CPL <= 4 ? 2 : 1;  // rows per batch: about 32 registers per buffer
    __shared__ float dots[2][ROUND_THREADS / 64][RB];
    __shared__ float inv_s;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int row0 = blockIdx.x * rows_per_wg;
    const int row_end = min(rows, row0 + rows_per_wg);
    v4f vv[CPL], acc[CPL];
    bool live[CPL];
#pragma unroll
    for (int k = 0; k < CPL; ++k) {
        const int col = 4 * tid + 4 * ROUND_THREADS * k;
        live[k] = col < cols;  // (cols is a multiple of 4)
        vv[k] = (!FIRST && live[k]) ? *reinterpret_cast<const v4f*>(v + col) : (v4f){0.f, 0.f, 0.f, 0.f};
        acc[k] = (v4f){0.f, 0.f, 0.f, 0.f};
    }
    if (w == 0) {
        float inv;
        if (FIRST) {
            inv = 1.0f / sqrtf((float)cols);
        } else {
            const float nrm = sqrtf(wave_total(ss_part, n_ss, lane));
            inv = nrm > 0.f ? 1.0f / nrm : 0.f;
        }
        if (lane == 0) inv_s = inv;
    }
    // (no branch around a load: rows beyond the workgroup's are read as its last row and get weight zero below,
    //  columns beyond the matrix are read as the row's first and get v = 0 / are masked, so that all loads of a
    //  batch are in flight together)
    auto load_batch = [&](v4f (&z)[RB][CPL], int r0) {
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            const int row = min(r0 + r, row_end - 1);
#pragma unroll
            for (int k = 0; k < CPL; ++k)
                z[r][k] = *reinterpret_cast<const v4f*>(Z + (size_t)row * cols + (live[k] ? 4 * tid + 4 * ROUND_THREADS * k : 0));
        }
    };
    auto abs4 = [](v4f a) { return (v4f){fabsf(a.x), fabsf(a.y), fabsf(a.z), fabsf(a.w)}; };
    v4f za[RB][CPL], zb[RB][CPL];
    load_batch(za, row0);
    int buf = 0;
    // (two batches per trip, so that the two register buffers keep their names)
    auto process = [&](v4f (&z)[RB][CPL], int r0) {
        float part[RB];
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            float sdot = 0.f;
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const v4f a = abs4(z[r][k]);
                if (FIRST) sdot += live[k] ? (a.x + a.y) + (a.z + a.w) : 0.f;
                else sdot += a.x * vv[k].x + a.y * vv[k].y + a.z * vv[k].z + a.w * vv[k].w;
            }
            part[r] = dbf_wave_sum_f(sdot);
        }
        if (lane == 0) {
#pragma unroll
            for (int r = 0; r < RB; ++r) dots[buf][w][r] = part[r];
        }
        __syncthreads();
        const float inv = inv_s;
#pragma unroll
        for (int r = 0; r < RB; ++r) {
            float tot = 0.f;
#pragma unroll
            for (int q = 0; q < ROUND_THREADS / 64; ++q) tot += dots[buf][q][r];
            const float ur = r0 + r < row_end ? tot * inv : 0.f;
            if (tid == r && r0 + r < row_end) u[r0 + r] = ur;
#pragma unroll
            for (int k = 0; k < CPL; ++k) {
                const v4f a = abs4(z[r][k]);
                acc[k].x += a.x * ur;  acc[k].y += a.y * ur;  acc[k].z += a.z * ur;  acc[k].w += a.w * ur;  // (dead columns: never stored)
            }
        }
        buf ^= 1;
    };
    for (int r0 = row0; r0 < row_end; r0 += 2 * RB) {
        load_batch(zb, r0 + RB);       // (rows beyond the workgroup's read as zeros without touching memory)
        process(za, r0);
        if (r0 + RB < row_end) {
            load_batch(za, r0 + 2 * RB);
            process(zb, r0 + RB);
        }
    }
#pragma unroll
    for (int k = 0; k < CPL; ++k)
        if (live[k]) *reinterpret_cast<v4f*>(partial + (size_t)blockIdx.x * cols + 4 * tid + 4 * ROUND_THREADS * k) = acc[k];
}

// partial[chunk][j] = sum over the chunk's rows i of |Z[i][j]| u[i]
__global__ __launch_bounds__(256) void dbf_svid_col_dots_kernel(const float* __restrict__ Z, int rows, int cols,
                                                               const float* __restrict__ u,
                                                               float* __restrict__ partial) {
    __shared__ float part[4][COL_BLOCK];
    const int cl = threadIdx.x & 63, rl = threadIdx.x >> 6;       // column quad, row lane
    const int col = blockIdx.x * COL_BLOCK + 4 * cl;
    const int row0 = blockIdx.y * COL_CHUNK_ROWS;
    float s[4] = {0.f, 0.f, 0.f, 0.f};
    const bool vec = (cols & 3) == 0 && col + 4 <= cols;
    if (vec) {
        // rows beyond the matrix are read as the last row with weight zero: no branch in the loop, so
        // the loads of several rounds are in flight together
        static_assert(COL_CHUNK_ROWS % 4 == 0, "four row lanes share a chunk evenly");
#pragma unroll
        for (int ii = 0; ii < COL_CHUNK_ROWS / 4; ++ii) {
            const int row = row0 + rl + 4 * ii;
            const int rc = min(row, rows - 1);
            const float w = row < rows ? u[rc] : 0.f;
            const v4f a = *reinterpret_cast<const v4f*>(Z + (size_t)rc * cols + col);
            s[0] += fabsf(a.x) * w;  s[1] += fabsf(a.y) * w;  s[2] += fabsf(a.z) * w;  s[3] += fabsf(a.w) * w;
        }
    } else {
        for (int i = rl; i < COL_CHUNK_ROWS; i += 4) {
            const int row = row0 + i;
            if (row >= rows) break;
            const float w = u[row];
            const float* z = Z + (size_t)row * cols + col;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (col + q < cols) s[q] += fabsf(z[q]) * w;
        }
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) part[rl][4 * cl + q] = s[q];
    __syncthreads();
    const int c = threadIdx.x;
    if (blockIdx.x * COL_BLOCK + c < cols)
        partial[(size_t)blockIdx.y * cols + blockIdx.x * COL_BLOCK + c] = ((part[0][c] + part[1][c]) + part[2][c]) + part[3][c];
}

// v_raw[j] = sum over chunks of partial[chunk][j]: four interleaved running sums (chunks c = 0, 4, 8, ... in the
// first, and so on), combined as ((s0 + s1) + s2) + s3; and ss_part[workgroup] = sum of v_raw[j]^2 over the
// workgroup's 64 columns (butterfly order).  Workgroup = 64 columns x the 4 running sums (one wavefront each: a
// thread's chain of dependent loads is a quarter of the chunks), combined through LDS in that fixed order.
__global__ __launch_bounds__(256) void dbf_svid_col_reduce_kernel(const float* __restrict__ partial, int chunks, int cols,
                                                               float* __restrict__ v, float* __restrict__ ss_part) {
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int j = blockIdx.x * 64 + lane;
    float s = 0.f;
    if (j < cols)
        for (int c = q; c < chunks; c += 4) s += partial[(size_t)c * cols + j];
    part[q][lane] = s;
    __syncthreads();
    if (q == 0) {
        const float vj = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
        if (j < cols) v[j] = vj;
        const float ss = wave_sum_f(vj * vj);
        if (lane == 0) ss_part[blockIdx.x] = ss;
    }
}

// The two factors from the unnormalised iterate: m = v_raw / ||v_raw|| (in place) and
// a = sigma u = u_raw ||v_raw|| / ||u_raw||^2 (sigma = ||v_raw|| / ||u_raw||, u = u_raw / ||u_raw||).
// Every workgroup forms both lengths itself, in the same fixed order, and then writes its 256 entries of each.
__global__ __launch_bounds__(256) void dbf_svid_finish_kernel(const float* __restrict__ u_raw, int rows,
                                                             const float* __restrict__ ss_part, int n_ss,
                                                             float* __restrict__ m, int cols, float* __restrict__ a) {
    __shared__ float part[256];
    float s = 0.f;
    for (int i = threadIdx.x; i < rows; i += 256) s += u_raw[i] * u_raw[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int w = 128; w >= 1; w >>= 1) {
        if ((int)threadIdx.x < w) part[threadIdx.x] += part[threadIdx.x + w];
        __syncthreads();
    }
    const float ssu = part[0];
    const float nv = sqrtf(wave_total(ss_part, n_ss, threadIdx.x & 63));
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < rows) a[i] = ssu > 0.f ? u_raw[i] * (nv / ssu) : 0.f;
    if (i < cols && nv > 0.f) m[i] = m[i] / nv;
}

// Sign(Z) into the tile layout: tile = 128 rows x 64 columns, byte 256 g + 16 r + j, bit s = sign of
// (row 16 s + r, column 16 g + j), a set bit meaning +1.  Thread t makes bytes 4t .. 4t+3.
__global__ __launch_bounds__(256) void dbf_svid_signs_kernel(const float* __restrict__ Z, int rows, int cols, int n_ct,
                                                            uint8_t* __restrict__ bits) {
    const int t = threadIdx.x;
    const int g = t >> 6, r = (t >> 2) & 15, j0 = 4 * (t & 3);
    const int col = blockIdx.x * DBF_TILE_COLS + 16 * g + j0;
    const bool vec = (cols & 3) == 0 && col + 4 <= cols;
    unsigned out = 0;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
        const int row = blockIdx.y * DBF_TILE_ROWS + 16 * s + r;
        if (row >= rows) continue;
        const float* z = Z + (size_t)row * cols + col;
        if (vec) {
            const v4f a = *reinterpret_cast<const v4f*>(z);
            out |= (unsigned)(a.x >= 0.f) << s;
            out |= (unsigned)(a.y >= 0.f) << (8 + s);
            out |= (unsigned)(a.z >= 0.f) << (16 + s);
            out |= (unsigned)(a.w >= 0.f) << (24 + s);
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q)
                if (col + q < cols) out |= (unsigned)(z[q] >= 0.f) << (8 * q + s);
        }
    }
    reinterpret_cast<unsigned*>(bits + ((size_t)blockIdx.y * n_ct + blockIdx.x) * DBF_TILE_BYTES)[t] = out;
}

inline size_t up256(size_t v) { return (v + 255) & ~(size_t)255; }
// Rows per workgroup of the one-pass round: one workgroup per compute unit (256 in all), at least 8 rows each.
inline int round_rows_per_wg(int rows) {
    const int per = (rows + 255) / 256;
    return per < 8 ? 8 : per;
}
template <int CPL>
void launch_round(bool first, int n_wg, hipStream_t st, const float* Z, int rows, int cols, const float* v,
                  const float* ss_part, int n_ss, float* u, float* partial, int rows_per_wg) {
    if (first)
        hipLaunchKernelGGL((dbf_svid_round_kernel<CPL, true>), dim3(n_wg), dim3(ROUND_THREADS), 0, st, Z, rows, cols, v, ss_part, n_ss,
                           u, partial, rows_per_wg);
    else
        hipLaunchKernelGGL((dbf_svid_round_kernel<CPL, false>), dim3(n_wg), dim3(ROUND_THREADS), 0, st, Z, rows, cols, v, ss_part, n_ss,
                           u, partial, rows_per_wg);
}
struct SvidWorkspace {
    size_t u, v, partial, scalars, total;
};
inline SvidWorkspace svid_workspace(int rows, int cols) {
    SvidWorkspace w;
    size_t chunks = ((size_t)rows + COL_CHUNK_ROWS - 1) / COL_CHUNK_ROWS;
    const size_t n_wg = ((size_t)rows + round_rows_per_wg(rows) - 1) / round_rows_per_wg(rows);
    if (n_wg > chunks) chunks = n_wg;  // partial sums: one row per 64-row chunk or per workgroup of the one-pass round
    size_t off = 0;
    w.u = off;        off = up256(off + 4 * (size_t)rows);
    w.v = off;        off = up256(off + 4 * (size_t)cols);
    w.partial = off;  off = up256(off + 4 * chunks * (size_t)cols);
    w.scalars = off;  off = up256(off + 4 * (((size_t)cols + 63) / 64));   // squared length of v_raw per 64 columns
    w.total = off;
    return w;
}

}  // namespace

extern "C" size_t dbf_svid_workspace_bytes(int rows, int cols) {
    if (rows < 1 || cols < 1 || rows > DBF_MAX_DIM || cols > DBF_MAX_DIM) return 0;
    return svid_workspace(rows, cols).total;
}

extern "C" int dbf_svid(const void* Z_dev, int rows, int cols, int iters, void* a_dev, void* m_dev, void* bits_dev,
                        void* workspace_dev, size_t workspace_bytes, void* hip_stream) {
    if (!Z_dev || !a_dev || !m_dev || !bits_dev || rows < 1 || cols < 1 || iters < 1) return DBF_EINVAL;
    if (rows > DBF_MAX_DIM || cols > DBF_MAX_DIM) return DBF_EINVAL;
    if ((reinterpret_cast<uintptr_t>(Z_dev) & 3) || (reinterpret_cast<uintptr_t>(a_dev) & 3) ||
        (reinterpret_cast<uintptr_t>(m_dev) & 3) || (reinterpret_cast<uintptr_t>(bits_dev) & 3))
        return DBF_EINVAL;
    const SvidWorkspace w = svid_workspace(rows, cols);
    if (!workspace_dev || (reinterpret_cast<uintptr_t>(workspace_dev) & 255) || workspace_bytes < w.total)
        return DBF_EWORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    const float* Z = static_cast<const float*>(Z_dev);
    uint8_t* base = static_cast<uint8_t*>(workspace_dev);
    float* u = reinterpret_cast<float*>(base + w.u);
    float* v = static_cast<float*>(m_dev);   // the right factor is iterated in place in the caller's buffer
    float* partial = reinterpret_cast<float*>(base + w.partial);
    float* ss_part = reinterpret_cast<float*>(base + w.scalars);
    const int vec_ok = ((cols & 3) == 0 && (reinterpret_cast<uintptr_t>(Z_dev) & 15) == 0 &&
                        (reinterpret_cast<uintptr_t>(m_dev) & 15) == 0) ? 1 : 0;
    const int chunks = (rows + COL_CHUNK_ROWS - 1) / COL_CHUNK_ROWS;
    const int n_rt = dbf_row_tiles(rows), n_ct = dbf_col_tiles(cols);
    const int n_ss = (cols + 63) / 64;

    hipLaunchKernelGGL(dbf_svid_signs_kernel, dim3(n_ct, n_rt), dim3(256), 0, st, Z, rows, cols, n_ct,
                       static_cast<uint8_t*>(bits_dev));
    const int cpl = (cols + 4 * ROUND_THREADS - 1) / (4 * ROUND_THREADS);  // float4s per thread and row in the one-pass round
    const int rpw = round_rows_per_wg(rows), n_wg = (rows + rpw - 1) / rpw;
    for (int it = 0; it < iters; ++it) {
        if (vec_ok && cpl <= 6 && (size_t)rows * cols >= ROUND_MIN_ENTRIES) {  // (7 float4s per thread and row spill)
            switch (cpl) {
                case 1: launch_round<1>(it == 0, n_wg, st, Z, rows, cols, v, ss_part, n_ss, u, partial, rpw); break;
                case 2: launch_round<2>(it == 0, n_wg, st, Z, rows, cols, v, ss_part, n_ss, u, partial, rpw); break;
                case 3: launch_round<3>(it == 0, n_wg, st, Z, rows, cols, v, ss_part, n_ss, u, partial, rpw); break;
                case 4: launch_round<4>(it == 0, n_wg, st, Z, rows, cols, v, ss_part, n_ss, u, partial, rpw); break;
                case 5: launch_round<5>(it == 0, n_wg, st, Z, rows, cols, v, ss_part, n_ss, u, partial, rpw); break;
                default: launch_round<6>(it == 0, n_wg, st, Z, rows, cols, v, ss_part, n_ss, u, partial, rpw); break;
            }
            hipLaunchKernelGGL(dbf_svid_col_reduce_kernel, dim3(n_ss), dim3(256), 0, st, partial, n_wg, cols, v, ss_part);
            continue;
        }
        if (it == 0)
            hipLaunchKernelGGL(dbf_svid_row_dots_kernel<true>, dim3((rows + 3) / 4), dim3(256), 0, st, Z, rows, cols, v,
                               ss_part, n_ss, u, vec_ok);
        else
            hipLaunchKernelGGL(dbf_svid_row_dots_kernel<false>, dim3((rows + 3) / 4), dim3(256), 0, st, Z, rows, cols, v,
                               ss_part, n_ss, u, vec_ok);
        hipLaunchKernelGGL(dbf_svid_col_dots_kernel, dim3((cols + COL_BLOCK - 1) / COL_BLOCK, chunks), dim3(256), 0, st,
                           Z, rows, cols, u, partial);
        hipLaunchKernelGGL(dbf_svid_col_reduce_kernel, dim3(n_ss), dim3(256), 0, st, partial, chunks, cols, v, ss_part);
    }
    const int longest = rows > cols ? rows : cols;
    hipLaunchKernelGGL(dbf_svid_finish_kernel, dim3((longest + 255) / 256), dim3(256), 0, st, u, rows, ss_part, n_ss, v,
                       cols, static_cast<float*>(a_dev));
    if (hipGetLastError() != hipSuccess) return DBF_EHIP;
    return DBF_OK;
}
