// Prediction head (Section 3.2): pooled vector -> perceptron d -> d_h (ReLU) -> n_out, then
// either the scalar itself (n_out == 1) or the expected value over K bins of Eq. 6.
//
// Layer 1 is a small [B x d] . [d x d_h] contraction kept entirely in fp32 (the pooled
// vector is never re-rounded); it is LDS-tiled, 64 x 64 outputs per workgroup, 4 x 4 per
// thread, and split along d (blockIdx.z) so that about a thousand workgroups exist even for one
// small batch; the splits leave partial pre-activations that layer 2 adds in split order
// (fixed order, bit-reproducible) before bias and ReLU.  Layer 2 and the K-bin decode are one
// workgroup per sequence.
#include "kernels.h"

namespace egtp {
namespace {

constexpr int TM = 64;  // head rows j per tile
constexpr int TN = 64;  // sequences per tile
constexpr int TK = 16;
constexpr int PAD = 4;

template <bool WBF16>
__global__ __launch_bounds__(256) void head_layer1_kernel(const float *__restrict__ x,
                                                          const int32_t *__restrict__ slot, int B, int d,
                                                          int d_h, const void *__restrict__ w1, int kchunk,
                                                          float *__restrict__ act_part)
{
    __shared__ float As[TK][TM + PAD];  // As[k][j]
    __shared__ float Bs[TK][TN + PAD];  // Bs[k][sequence]
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int j0 = blockIdx.x * TM, s0 = blockIdx.y * TN;

    const int lrow = tid >> 2;
    const int lk = (tid & 3) * 4;
    int jrow = j0 + lrow;
    jrow = jrow < d_h ? jrow : d_h - 1;  // clamped rows are computed and dropped
    int srow = s0 + lrow;
    srow = srow < B ? srow : B - 1;
    const long xrow = slot ? slot[srow] : srow;
    const float *xp = x + xrow * (long)d;

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            acc[i][j] = 0.f;

    const int kbeg = blockIdx.z * kchunk;
    const int kend = min(d, kbeg + kchunk);
    float *act = act_part + (long)blockIdx.z * B * d_h;
    for (int k0 = kbeg; k0 < kend; k0 += TK) {
        float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
        if (k0 + lk < kend) {
            if (WBF16) {
                const uint2 q = *(const uint2 *)((const unsigned short *)w1 + (long)jrow * d + k0 + lk);
                a.x = __uint_as_float(q.x << 16);
                a.y = __uint_as_float(q.x & 0xffff0000u);
                a.z = __uint_as_float(q.y << 16);
                a.w = __uint_as_float(q.y & 0xffff0000u);
            } else {
                a = *(const float4 *)((const float *)w1 + (long)jrow * d + k0 + lk);
            }
            b = *(const float4 *)(xp + k0 + lk);
        }
        __syncthreads();
        As[lk + 0][lrow] = a.x;
        As[lk + 1][lrow] = a.y;
        As[lk + 2][lrow] = a.z;
        As[lk + 3][lrow] = a.w;
        Bs[lk + 0][lrow] = b.x;
        Bs[lk + 1][lrow] = b.y;
        Bs[lk + 2][lrow] = b.z;
        Bs[lk + 3][lrow] = b.w;
        __syncthreads();
#pragma unroll
        for (int k = 0; k < TK; ++k) {
            const float4 av = *(const float4 *)&As[k][tx * 4];
            const float4 bv = *(const float4 *)&Bs[k][ty * 4];
            const float aa[4] = {av.x, av.y, av.z, av.w};
            const float bb[4] = {bv.x, bv.y, bv.z, bv.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = fmaf(aa[i], bb[j], acc[i][j]);
        }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int s = s0 + ty * 4 + j;
        if (s >= B)
            continue;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int jj = j0 + tx * 4 + i;
            if (jj < d_h)
                act[(long)s * d_h + jj] = acc[i][j];
        }
    }
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1)
        v += __shfl_xor(v, o);
    return v;
}

// one workgroup (4 waves) per sequence: out[o] = b2[o] + w2[o,:] . act[b,:]; n_out > 1 => Eq. 6
// LDS: a[d_h] | partial[4][n_out]
template <bool WBF16>
__global__ __launch_bounds__(256) void head_layer2_kernel(const float *__restrict__ act_part, int nks, int B,
                                                          const float *__restrict__ b1, int d_h, int n_out,
                                                          const void *__restrict__ w2,
                                                          const float *__restrict__ b2,
                                                          const float *__restrict__ centers,
                                                          float *__restrict__ pred)
{
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    extern __shared__ float a[];
    float *partial = a + d_h;
    // hidden activations: partial sums in split order, then bias and ReLU; kept in LDS
    for (int j = tid; j < d_h; j += 256) {
        float pre = 0.f;
#pragma unroll 8
        for (int z = 0; z < nks; ++z)
            pre += act_part[((long)z * B + b) * d_h + j];
        pre += b1 ? b1[j] : 0.f;
        a[j] = pre > 0.f ? pre : 0.f;
    }
    __syncthreads();
    // every wave takes a quarter of each dot product (fixed assignment: bit-reproducible)
    for (int o = 0; o < n_out; ++o) {
        float s = 0.f;
#pragma unroll 4
        for (int j = tid; j < d_h; j += 256) {
            float w;
            if (WBF16)
                w = __uint_as_float((unsigned)((const unsigned short *)w2)[(long)o * d_h + j] << 16);
            else
                w = ((const float *)w2)[(long)o * d_h + j];
            s = fmaf(w, a[j], s);
        }
        s = wave_sum(s);
        if (lane == 0)
            partial[wave * n_out + o] = s;
    }
    __syncthreads();
    if (wave != 0)
        return;
    // online softmax-expectation over the n_out outputs (every lane carries the same values)
    float m = -__builtin_inff(), den = 0.f, num = 0.f, y = 0.f;
    for (int o = 0; o < n_out; ++o) {
        const float s = ((partial[o] + partial[n_out + o]) + (partial[2 * n_out + o] + partial[3 * n_out + o])) +
                        (b2 ? b2[o] : 0.f);
        if (n_out == 1) {
            y = s;
        } else {
            const float mn = fmaxf(m, s);
            const float sc = __expf(m - mn);  // exp(-inf) = 0 on the first bin
            const float e = __expf(s - mn);
            den = den * sc + e;
            num = num * sc + e * centers[o];
            m = mn;
        }
    }
    if (lane == 0)
        pred[b] = n_out == 1 ? y : num / den;
}

}  // namespace

int head_k_splits(int d, int d_h, int32_t B)
{
    int base = (d + 511) / 512;  // slices of at most 512 along d ...
    base = base < 1 ? 1 : (base > 8 ? 8 : base);
    const long tiles = (long)((d_h + TM - 1) / TM) * ((B + TN - 1) / TN);
    long want = tiles > 0 ? (1024 + tiles - 1) / tiles : 1;  // ... thinner when the batch has few tiles
    const int cap = (d + TK - 1) / TK < 64 ? (d + TK - 1) / TK : 64;
    long n = want > base ? want : base;
    n = n > cap ? cap : n;
    return n < 1 ? 1 : (int)n;
}

size_t head_act_floats_bound(int d, int d_h, int32_t B)
{
    // the number of planes only depends on how many 64-sequence tiles the batch has
    size_t best = 0;
    for (int32_t st = 1; st <= (B + TN - 1) / TN; ++st) {
        const int32_t b = st * TN < B ? st * TN : B;
        const size_t f = (size_t)head_k_splits(d, d_h, b) * (size_t)b * (size_t)d_h;
        best = f > best ? f : best;
    }
    return best;
}

hipError_t head_layer1(const float *x, const int32_t *slot, int32_t B, int d, int d_h, const void *w1,
                       int wdtype, float *act_part, hipStream_t st)
{
    if (B <= 0)
        return hipSuccess;
    const int nks = head_k_splits(d, d_h, B);
    const int kchunk = ((d + nks - 1) / nks + TK - 1) / TK * TK;  // multiple of the K step
    const dim3 grid((d_h + TM - 1) / TM, (B + TN - 1) / TN, nks);
    if (wdtype == DT_BF16)
        hipLaunchKernelGGL(head_layer1_kernel<true>, grid, dim3(256), 0, st, x, slot, B, d, d_h, w1, kchunk,
                           act_part);
    else
        hipLaunchKernelGGL(head_layer1_kernel<false>, grid, dim3(256), 0, st, x, slot, B, d, d_h, w1, kchunk,
                           act_part);
    return hipGetLastError();
}

hipError_t head_forward(const HeadArgs &a, hipStream_t st)
{
    if (a.B <= 0)
        return hipSuccess;
    const int nks = head_k_splits(a.d, a.d_h, a.B);
    const size_t lds2 = ((size_t)a.d_h + 4 * (size_t)a.n_out) * sizeof(float);
    if (lds2 > 96 * 1024)
        return hipErrorInvalidValue;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e1 = hipFuncSetAttribute((const void *)head_layer2_kernel<true>,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        hipError_t e2 = hipFuncSetAttribute((const void *)head_layer2_kernel<false>,
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
        if (e1 != hipSuccess || e2 != hipSuccess)
            return e1 != hipSuccess ? e1 : e2;
        attr_set = true;
    }
    hipError_t e = head_layer1(a.x, a.slot, a.B, a.d, a.d_h, a.w1, a.wdtype, a.act, st);
    if (e != hipSuccess)
        return e;
    if (a.wdtype == DT_BF16)
        hipLaunchKernelGGL(head_layer2_kernel<true>, dim3(a.B), dim3(256), lds2, st, a.act, nks, a.B, a.b1, a.d_h,
                           a.n_out, a.w2, a.b2, a.bin_centers, a.pred);
    else
        hipLaunchKernelGGL(head_layer2_kernel<false>, dim3(a.B), dim3(256), lds2, st, a.act, nks, a.B, a.b1, a.d_h,
                           a.n_out, a.w2, a.b2, a.bin_centers, a.pred);
    return hipGetLastError();
}

}  // namespace egtp
