// Wave-wide (64 lanes) reductions by a fixed xor tree: every lane ends up with the result, and the
// order of the additions is the same in every run.  Device-side header.
#pragma once
#include <hip/hip_runtime.h>

namespace egtp {
namespace {

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o);
    return v;
}

__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

}  // namespace
}  // namespace egtp
