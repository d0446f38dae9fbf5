// Streaming-read probe: how fast can this GPU pull bytes from HBM with the same 16-byte
// per-lane loads the decode kernels use, and no arithmetic to speak of?  The result is the
// practical ceiling the decode kernels are compared with, next to the 8 TB/s data-sheet peak.
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

}  // namespace

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
