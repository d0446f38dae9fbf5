// Streaming-read probe: how fast can this GPU pull bytes from HBM with the same 16-byte
// per-lane loads the decode kernels use, and no arithmetic to speak of?  The result is the
// practical ceiling the decode kernels are compared with, next to the 8 TB/s data-sheet peak.
//
// Matrix-pipe probe: int8 matrix instructions on independent accumulators, with or without the
// ANDs that turn sign bytes into an operand (one per operand register, as the prefill kernel does
// them), and nothing else: what the matrix pipe sustains next to its 5.0 POP/s data-sheet peak.
#include <type_traits>

#include "dbf_kernels.h"

namespace {

typedef unsigned int v4u __attribute__((ext_vector_type(4)));

constexpr int PROBE_LOADS = 16;                          // 16-byte loads in flight per lane
constexpr int PROBE_WG_BYTES = 256 * 16 * PROBE_LOADS;   // 64 KiB per workgroup

__global__ __launch_bounds__(256) void dbf_probe_read_kernel(const v4u* __restrict__ src,
                                                             unsigned* __restrict__ sink) {
    const v4u* p = src + (size_t)blockIdx.x * (PROBE_WG_BYTES / 16) + threadIdx.x;
    v4u v[PROBE_LOADS];
#pragma unroll
    for (int i = 0; i < PROBE_LOADS; ++i) v[i] = __builtin_nontemporal_load(p + i * 256);
    unsigned acc = 0;
#pragma unroll
    for (int i = 0; i < PROBE_LOADS; ++i) acc ^= v[i].x ^ v[i].y ^ v[i].z ^ v[i].w;
    if (acc == 0x9E3779B9u && sink) *sink = acc;  // keeps the loads alive; practically never taken
}

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// WIDE = false: v_mfma_i32_16x16x64_i8 (4 passes), 32 accumulators; true: v_mfma_i32_32x32x32_i8
// (8 passes), 8 accumulators: 128 accumulator registers either way, 2^19 resp. 2^18 multiply-adds per
// iteration.  GROUP = matrix instructions that share one masked operand (4 ANDs); 0 = no ANDs.
template <bool WIDE, int GROUP>
__global__ __launch_bounds__(256) void dbf_probe_mfma_kernel(int iters, unsigned seed, int* __restrict__ sink) {
    constexpr int NACC = WIDE ? 8 : 32, G = GROUP ? GROUP : NACC;
    typedef typename std::conditional<WIDE, v16i, v4i>::type acc_t;
    acc_t acc[NACC];
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int j = 0; j < (WIDE ? 16 : 4); ++j) acc[i][j] = 0;
    const v4i x = {(int)seed, (int)seed * 3, (int)seed * 5, (int)seed * 7};
    unsigned b0 = seed ^ threadIdx.x, b1 = b0 * 3u, b2 = b0 * 5u, b3 = b0 * 7u;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int g = 0; g < NACC / G; ++g) {
            const unsigned m = GROUP ? 0x01010101u << (g & 7) : 0xFFFFFFFFu;
            const v4i a = {(int)(b0 & m), (int)(b1 & m), (int)(b2 & m), (int)(b3 & m)};
#pragma unroll
            for (int t = 0; t < G; ++t) {
                if constexpr (WIDE) acc[G * g + t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, x, acc[G * g + t], 0, 0, 0);
                else acc[G * g + t] = __builtin_amdgcn_mfma_i32_16x16x64_i8(a, x, acc[G * g + t], 0, 0, 0);
            }
        }
        b0 += 0x01010101u;
    }
    int r = 0;
#pragma unroll
    for (int i = 0; i < NACC; ++i)
#pragma unroll
        for (int j = 0; j < (WIDE ? 16 : 4); ++j) r += acc[i][j];
    if (r == 0x12345678 && sink) *sink = r;  // keeps the arithmetic alive; practically never taken
}

}  // namespace

extern "C" int dbf_probe_mfma(int wide, int with_ands, int wavefronts_per_simd, int iters, void* sink_dev,
                              void* hip_stream, double* ops) {
    if (wavefronts_per_simd < 1 || wavefronts_per_simd > 4 || iters < 1) return DBF_EINVAL;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        return DBF_EHIP;
    const dim3 grid((unsigned)(cus * wavefronts_per_simd)), block(256);  // one wavefront per SIMD per workgroup
    hipStream_t st = static_cast<hipStream_t>(hip_stream);
    int* sink = static_cast<int*>(sink_dev);
    if (wide) {
        if (with_ands) hipLaunchKernelGGL((dbf_probe_mfma_kernel<true, 2>), grid, block, 0, st, iters, 12345u, sink);
        else hipLaunchKernelGGL((dbf_probe_mfma_kernel<true, 0>), grid, block, 0, st, iters, 12345u, sink);
    } else {
        if (with_ands) hipLaunchKernelGGL((dbf_probe_mfma_kernel<false, 4>), grid, block, 0, st, iters, 12345u, sink);
        else hipLaunchKernelGGL((dbf_probe_mfma_kernel<false, 0>), grid, block, 0, st, iters, 12345u, sink);
    }
    if (hipGetLastError() != hipSuccess) return DBF_EHIP;
    // per wavefront and iteration: 32 x (16*16*64) or 8 x (32*32*32) multiply-adds, two operations each
    if (ops) *ops = (wide ? 524288.0 : 1048576.0) * iters * 4.0 * grid.x;
    return DBF_OK;
}

extern "C" int dbf_probe_read(const void* src_dev, size_t bytes, void* sink_dev, void* hip_stream) {
    if (!src_dev || bytes < (size_t)PROBE_WG_BYTES) return DBF_EINVAL;
    if (reinterpret_cast<uintptr_t>(src_dev) & 15) return DBF_EINVAL;
    const size_t blocks = bytes / PROBE_WG_BYTES;  // the tail beyond a multiple of 64 KiB is not read
    if (blocks > 0x7FFFFFFFull) return DBF_EINVAL;
    hipLaunchKernelGGL(dbf_probe_read_kernel, dim3((unsigned)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(hip_stream), static_cast<const v4u*>(src_dev),
                       static_cast<unsigned*>(sink_dev));
    if (hipGetLastError() != hipSuccess) return DBF_EHIP;
    return DBF_OK;
}
