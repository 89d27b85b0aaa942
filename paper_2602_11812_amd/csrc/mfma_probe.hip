// Measurement aid: the rate the bf16 matrix cores sustain when nothing but MFMAs run -- operands
// and accumulators stay in registers, no memory traffic -- in the same shape, tile order and
// occupancy as the fused LM-head + entropy kernel (Eq. 2): one wave per SIMD, an 8 x 8 grid of
// 16x16x32 MFMAs per step, first operand held for eight MFMAs in a row.  With all-zero operands
// this is the clock-limited rate; with random operands the package power limit sets it.
#include "kernels.h"

namespace egtp {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ unsigned mix32(unsigned x)
{
    x ^= x >> 16;
    x *= 0x7feb352dU;
    x ^= x >> 15;
    x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}

// eight values in [-1, 1) from a counter, or eight zeros
__device__ bf16x8 probe_fragment(unsigned counter, int random_operands)
{
    bf16x8 f;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const unsigned h = mix32(counter * 8u + (unsigned)i);
        const float v = random_operands ? (float)(h & 0xffffu) * (1.0f / 32768.0f) - 1.0f : 0.0f;
        f[i] = (__bf16)v;
    }
    return f;
}

__global__ __launch_bounds__(256, 1) void mfma_probe_kernel(float *__restrict__ sink, int iters,
                                                            int random_operands)
{
    const unsigned tid = blockIdx.x * 256u + threadIdx.x;
    bf16x8 a[8], b[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = probe_fragment(tid * 16u + (unsigned)i, random_operands);
        b[i] = probe_fragment(tid * 16u + 8u + (unsigned)i, random_operands);
    }
    f32x4 c[8][8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
            c[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
#pragma unroll
            for (int j = 0; j < 8; ++j)
                c[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i], b[j], c[i][j], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int j = 0; j < 8; ++j)
            sum += c[i][j][0] + c[i][j][1] + c[i][j][2] + c[i][j][3];
    sink[tid] = sum;  // keeps the loop alive
}

}  // namespace

double mfma_probe_flop(int iters)
{
    // workgroups x waves x steps x MFMAs per step x (16 * 16 * 32 multiply-adds)
    return (double)MFMA_PROBE_WORKGROUPS * 4.0 * (double)iters * 64.0 * (2.0 * 16 * 16 * 32);
}

hipError_t mfma_probe_launch(float *sink, int iters, int random_operands, hipStream_t st)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3(MFMA_PROBE_WORKGROUPS), dim3(256), 0, st, sink, iters,
                       random_operands);
    return hipGetLastError();
}

}  // namespace egtp
