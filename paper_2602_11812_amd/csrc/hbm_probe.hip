// Measurement aid: the rate at which the device streams a large buffer out of HBM with plain
// 16-byte-per-lane loads and nothing else to do -- the ceiling that the pooling kernels (Eq. 4, which
// read every hidden state once more) can be set against beside the published peak.  The loads carry
// the non-temporal hint, like the pooling kernels' own: data that is read once should not displace
// anything in the caches, and on this part the hint alone is worth a tenth of the bandwidth (measured:
// 5.9 TB/s without, 6.4 - 6.6 TB/s with it, workgroups reading contiguous slabs).
#include "kernels.h"
#include "stream_load.h"

namespace egtp {
namespace {

constexpr int PROBE_IN_FLIGHT = 8;  // 16-byte loads a thread has outstanding

// Workgroup w streams the w-th contiguous slab of the buffer; a wave reads 1 KiB at a time.
__global__ __launch_bounds__(256) void hbm_read_probe_kernel(const u32x4 *__restrict__ src, size_t n16,
                                                             unsigned *__restrict__ sink)
{
    const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per_wg;
    const size_t hi = lo + per_wg < n16 ? lo + per_wg : n16;
    unsigned acc = 0;
    size_t i = lo + threadIdx.x;
    for (; i + (size_t)(PROBE_IN_FLIGHT - 1) * 256 < hi; i += (size_t)PROBE_IN_FLIGHT * 256) {
        u32x4 q[PROBE_IN_FLIGHT];
#pragma unroll
        for (int j = 0; j < PROBE_IN_FLIGHT; ++j)
            q[j] = stream_load16(src + i + (size_t)j * 256);
#pragma unroll
        for (int j = 0; j < PROBE_IN_FLIGHT; ++j)
            acc ^= q[j].x ^ q[j].y ^ q[j].z ^ q[j].w;
    }
    for (; i < hi; i += 256) {
        const u32x4 q = stream_load16(src + i);
        acc ^= q.x ^ q.y ^ q.z ^ q.w;
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;  // keeps the loads alive
}

}  // namespace

hipError_t hbm_read_probe_launch(const void *buf, size_t bytes, unsigned *sink, hipStream_t st)
{
    hipLaunchKernelGGL(hbm_read_probe_kernel, dim3(HBM_PROBE_WORKGROUPS), dim3(256), 0, st, (const u32x4 *)buf,
                       bytes / 16, sink);
    return hipGetLastError();
}

}  // namespace egtp
