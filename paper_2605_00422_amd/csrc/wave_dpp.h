// Reductions over the 64 lanes of a wavefront on DPP row operations: no LDS traffic, wave-uniform results.
#pragma once
#include "bwla_internal.h"

namespace {

template <int CTRL>
__device__ __forceinline__ int dl_dpp(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true);
}
// largest of non-negative floats over the wavefront, as a wave-uniform value
__device__ __forceinline__ float dl_wave_max_nonneg(float v) {
    int x = __float_as_int(v);                         // non-negative floats order like their bits
    x = max(x, dl_dpp<0xB1>(x));                       // quad_perm [1,0,3,2]
    x = max(x, dl_dpp<0x4E>(x));                       // quad_perm [2,3,0,1]
    x = max(x, dl_dpp<0x141>(x));                      // row_half_mirror
    x = max(x, dl_dpp<0x140>(x));                      // row_mirror: every lane of a row of 16 has the row's maximum
    const int r0 = __builtin_amdgcn_readlane(x, 0), r1 = __builtin_amdgcn_readlane(x, 16);
    const int r2 = __builtin_amdgcn_readlane(x, 32), r3 = __builtin_amdgcn_readlane(x, 48);
    return __int_as_float(max(max(r0, r1), max(r2, r3)));
}
__device__ __forceinline__ int dl_wave_sum(int x) {
    x += dl_dpp<0xB1>(x);
    x += dl_dpp<0x4E>(x);
    x += dl_dpp<0x141>(x);
    x += dl_dpp<0x140>(x);
    return __builtin_amdgcn_readlane(x, 0) + __builtin_amdgcn_readlane(x, 16) + __builtin_amdgcn_readlane(x, 32) +
           __builtin_amdgcn_readlane(x, 48);
}

}  // namespace
