// Wavefront-wide reductions shared by the HIP kernels of libdbf (device code only).
#ifndef DBF_WAVE_H
#define DBF_WAVE_H

#include <hip/hip_runtime.h>

// Reductions with data-parallel-primitive moves (register to register, a few cycles each) instead of
// LDS-crossbar shuffles (~100 cycles each, six in a chain): butterflies inside every row of 16 lanes, then
// the four row results through scalar registers.
template <int CTRL>
__device__ inline int dbf_dpp_move(int v) {
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}
__device__ inline float dbf_wave_max(float v) {
    v = fmaxf(v, __builtin_bit_cast(float, dbf_dpp_move<0xB1>(__builtin_bit_cast(int, v))));   // quad_perm [1,0,3,2]
    v = fmaxf(v, __builtin_bit_cast(float, dbf_dpp_move<0x4E>(__builtin_bit_cast(int, v))));   // quad_perm [2,3,0,1]
    v = fmaxf(v, __builtin_bit_cast(float, dbf_dpp_move<0x124>(__builtin_bit_cast(int, v))));  // row_ror:4
    v = fmaxf(v, __builtin_bit_cast(float, dbf_dpp_move<0x128>(__builtin_bit_cast(int, v))));  // row_ror:8
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}
__device__ inline int dbf_wave_sum(int v) {
    v += dbf_dpp_move<0xB1>(v);
    v += dbf_dpp_move<0x4E>(v);
    v += dbf_dpp_move<0x124>(v);
    v += dbf_dpp_move<0x128>(v);
    return __builtin_amdgcn_readlane(v, 0) + __builtin_amdgcn_readlane(v, 16) + __builtin_amdgcn_readlane(v, 32) +
           __builtin_amdgcn_readlane(v, 48);
}

// Sum of a float over the wavefront, the same value in every lane: each row of 16 lanes is summed by its
// lane 0 in a fixed tree, the four row sums are added as (r0 + r1) + (r2 + r3).
__device__ inline float dbf_wave_sum_f(float v) {
    v += __builtin_bit_cast(float, dbf_dpp_move<0xB1>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, dbf_dpp_move<0x4E>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, dbf_dpp_move<0x124>(__builtin_bit_cast(int, v)));
    v += __builtin_bit_cast(float, dbf_dpp_move<0x128>(__builtin_bit_cast(int, v)));
    const int b = __builtin_bit_cast(int, v);
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return (r0 + r1) + (r2 + r3);
}

#endif  // DBF_WAVE_H
