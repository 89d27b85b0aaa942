// Layer 1 of a prediction head is split along d into slices that leave partial pre-activations in planes
// act_part[slice][sequence][d_h].  Consumers run one workgroup per sequence, for which adding the planes up is a
// chain of memory latencies: PLANES_AHEAD planes are fetched before any is used, four neighbouring outputs per
// thread (one 16-byte load per plane).  The planes are added in slice order: bit-reproducible.  Device-side header.
#pragma once
#include <hip/hip_runtime.h>

namespace egtp {

constexpr int PLANES_AHEAD = 16;

// sum over the nks planes of outputs j .. j + 3 of sequence b; needs d_h % 4 == 0 and j % 4 == 0
__device__ __forceinline__ float4 sum_planes4(const float *__restrict__ act_part, int nks, int B, int b, int d_h, int j)
{
    float4 pre = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int s0 = 0; s0 < nks; s0 += PLANES_AHEAD) {
        float4 v[PLANES_AHEAD];
#pragma unroll
        for (int i = 0; i < PLANES_AHEAD; ++i) {
            const int s = s0 + i < nks ? s0 + i : nks - 1;  // past the end: a valid plane, not used
            v[i] = *(const float4 *)(act_part + ((long)s * B + b) * d_h + j);
        }
#pragma unroll
        for (int i = 0; i < PLANES_AHEAD; ++i)
            if (s0 + i < nks)
                pre.x += v[i].x, pre.y += v[i].y, pre.z += v[i].z, pre.w += v[i].w;
    }
    return pre;
}

}  // namespace egtp
