// Cross-lane helpers shared by the kernels (64-lane wavefronts): a lane reads a register of
// another lane through ds_bpermute (no LDS memory involved), and a value every lane holds
// identically is moved to scalar registers.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace ntp {

__device__ __forceinline__ int bperm_i(int src_lane, int v) {
    return __builtin_amdgcn_ds_bpermute(src_lane << 2, v);
}
__device__ __forceinline__ float bperm_f(int src_lane, float v) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src_lane << 2, __float_as_int(v)));
}
__device__ __forceinline__ int64_t uniform64(int64_t v) {
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)(v & 0xffffffff));
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)((uint64_t)v >> 32));
    return (int64_t)(((uint64_t)hi << 32) | lo);
}

}  // namespace ntp
