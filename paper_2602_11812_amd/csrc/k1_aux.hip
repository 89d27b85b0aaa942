// Kernels around the fused entropy kernel (Eq. 2): packing of row-major operands (bf16 as they are, fp32
// as six K segments of bf16 pieces) into the block layout the fused kernel reads, and the merge of its
// partial statistics into H.
#include "bf16_split.h"
#include "k1_common.h"

namespace egtp {
namespace {

// entropy[t] from the nsplit partial triples of token t, merged in range order
__global__ __launch_bounds__(256) void k1_merge_kernel(const float *__restrict__ part, int nsplit,
                                                       long T, float *__restrict__ entropy)
{
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= T)
        return;
    const long plane = (long)nsplit * T;
    Stats a;
    a.m = part[t];
    a.S = part[plane + t];
    a.U = part[2 * plane + t];
    for (int s = 1; s < nsplit; ++s) {
        Stats b;
        const long idx = (long)s * T + t;
        b.m = part[idx];
        b.S = part[plane + idx];
        b.U = part[2 * plane + idx];
        a = merge(a, b);
    }
    entropy[t] = logf(a.S) - a.U * 0.6931471805599453f / a.S;
}

// The same merge for many ranges per token (small batches split the vocabulary finely).
// Workgroup = 8 tokens x 32 groups: thread (token, g) merges ranges g, g+32, ... in order, then the
// 32 groups of a token are joined by a fixed xor tree inside each wave and through LDS across the
// four waves.  A fixed order, so bit-reproducible.
// The triples of 8 ranges are fetched before any of them is merged: the kernel is a chain of
// cache misses otherwise.
constexpr int WIDE_TOKENS = 8, WIDE_GROUPS = 32, WIDE_BATCH = 8;
__global__ __launch_bounds__(256) void k1_merge_wide_kernel(const float *__restrict__ part, int nsplit,
                                                            long T, float *__restrict__ entropy)
{
    __shared__ float red[4][WIDE_TOKENS][3];
    const int tl = threadIdx.x & (WIDE_TOKENS - 1);
    const int g = threadIdx.x / WIDE_TOKENS;
    const long t = (long)blockIdx.x * WIDE_TOKENS + tl;
    const long plane = (long)nsplit * T;
    Stats a;
    a.m = NEG_BIG;
    a.S = 0.f;
    a.U = 0.f;
    if (t < T) {
        for (int s0 = g; s0 < nsplit; s0 += WIDE_GROUPS * WIDE_BATCH) {
            Stats b[WIDE_BATCH];
#pragma unroll
            for (int i = 0; i < WIDE_BATCH; ++i) {
                const int s = s0 + i * WIDE_GROUPS;
                const long idx = (long)(s < nsplit ? s : g) * T + t;  // past the end: any valid range, unused
                b[i].m = part[idx];
                b[i].S = part[plane + idx];
                b[i].U = part[2 * plane + idx];
            }
#pragma unroll
            for (int i = 0; i < WIDE_BATCH; ++i)
                if (s0 + i * WIDE_GROUPS < nsplit)
                    a = merge(a, b[i]);
        }
    }
    // join the 8 groups of a wave (lanes 8, 16, 32 apart), then the 4 waves through LDS
#pragma unroll
    for (int o = WIDE_TOKENS; o < 64; o <<= 1) {
        Stats b;
        b.m = __shfl_xor(a.m, o);
        b.S = __shfl_xor(a.S, o);
        b.U = __shfl_xor(a.U, o);
        a = merge(a, b);
    }
    const int wave = threadIdx.x >> 6;
    if ((threadIdx.x & 63) < WIDE_TOKENS) {
        red[wave][tl][0] = a.m;
        red[wave][tl][1] = a.S;
        red[wave][tl][2] = a.U;
    }
    __syncthreads();
    if (threadIdx.x < WIDE_TOKENS && t < T) {
#pragma unroll
        for (int k = 1; k < 4; ++k) {
            Stats b;
            b.m = red[k][tl][0];
            b.S = red[k][tl][1];
            b.U = red[k][tl][2];
            a = merge(a, b);
        }
        entropy[t] = logf(a.S) - a.U * 0.6931471805599453f / a.S;
    }
}

// Packs rows of a row-major bf16 matrix src[R x d] into blocks of 256 rows x 32 K-elements in
// LDS-image order; rows >= R and K >= d are zero.  One workgroup packs 8 consecutive K steps
// of `rows_per_wg` rows (a multiple of 8; blockIdx.z picks the row group) of one row tile: a wave
// reads 512 contiguous bytes of each of two rows at a time.
__global__ __launch_bounds__(256) void pack_rows_bf16_kernel(const unsigned char *__restrict__ src, long R,
                                                             int d, int KT, int rows_per_wg,
                                                             unsigned char *__restrict__ dst)
{
    const long tile = blockIdx.x;
    const int ks0 = blockIdx.y * 8;
    const int c32 = threadIdx.x & 31;   // 16-byte chunk of the 512-byte span: K step c32/4, chunk c32%4
    const int rsub = threadIdx.x >> 5;  // 8 rows per pass
    const int ks = ks0 + (c32 >> 2);
    const int chunk = c32 & 3;
    const long k_elem = (long)ks * BK + chunk * 8;
    if (ks >= KT)
        return;
    unsigned char *blk = dst + (tile * KT + ks) * (long)TILE_BYTES;
    const int r0 = blockIdx.z * rows_per_wg;
    for (int r = r0 + rsub; r < r0 + rows_per_wg; r += 8) {
        const long row = tile * 256 + r;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < R && k_elem < d)
            v = *(const uint4 *)(src + (row * d + k_elem) * 2);
        *(uint4 *)(blk + r * ROW_BYTES + ((chunk ^ swizzle_key(r)) << 4)) = v;
    }
}

// fp32 operands.  With w = w0 + w1 + w2 and h = h0 + h1 + h2 (bf16 pieces, leading piece first), w.h is
// the sum of nine piece products of relative size 2^-8(i+j); the three smallest (i + j >= 3, below
// 2^-24) are dropped, and the other six are laid side by side along K -- one bf16 contraction of length
// 6 * dseg, dseg = d rounded up to whole 32-element blocks.  Segment s multiplies piece SPLIT_W[s] of W_lm
// with piece SPLIT_H[s] of the hidden state; the smallest products come first, so the fp32 accumulators
// meet the terms in ascending order of magnitude.
__device__ constexpr int SPLIT_W[K1_SPLIT_TERMS] = {2, 1, 0, 1, 0, 0};
__device__ constexpr int SPLIT_H[K1_SPLIT_TERMS] = {0, 1, 2, 0, 1, 0};

// Packs rows of a row-major fp32 matrix src[R x d] (d % 4 == 0) into the six segments of one operand
// side.  Thread layout as in the bf16 kernel, over the `kseg` blocks of ONE segment: every thread reads
// its 8 values once, splits them, and stores the piece each segment asks for.
template <bool HIDDEN_SIDE>
__global__ __launch_bounds__(256) void pack_rows_f32_split_kernel(const float *__restrict__ src, long R, int d,
                                                                  int kseg, int rows_per_wg,
                                                                  unsigned char *__restrict__ dst)
{
    const long tile = blockIdx.x;
    const int c32 = threadIdx.x & 31;
    const int rsub = threadIdx.x >> 5;
    const int kk = blockIdx.y * 8 + (c32 >> 2);  // block inside a segment
    const int chunk = c32 & 3;
    if (kk >= kseg)
        return;
    const long k_elem = (long)kk * BK + chunk * 8;
    const long KT = (long)K1_SPLIT_TERMS * kseg;
    const int r0 = blockIdx.z * rows_per_wg;
    for (int r = r0 + rsub; r < r0 + rows_per_wg; r += 8) {
        const long row = tile * 256 + r;
        float4 lo4 = make_float4(0.f, 0.f, 0.f, 0.f), hi4 = lo4;
        if (row < R) {  // d % 4 == 0: a group of four lies wholly inside a row or wholly past its end
            if (k_elem < d)
                lo4 = *(const float4 *)(src + row * d + k_elem);
            if (k_elem + 4 < d)
                hi4 = *(const float4 *)(src + row * d + k_elem + 4);
        }
        const float f[8] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
        unsigned pc[3][8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            split3_bits(f[i], pc[0][i], pc[1][i], pc[2][i]);
        uint4 q[3];
#pragma unroll
        for (int p = 0; p < 3; ++p)
            q[p] = make_uint4((pc[p][0] >> 16) | pc[p][1], (pc[p][2] >> 16) | pc[p][3], (pc[p][4] >> 16) | pc[p][5],
                              (pc[p][6] >> 16) | pc[p][7]);
        const int in_block = r * ROW_BYTES + ((chunk ^ swizzle_key(r)) << 4);
#pragma unroll
        for (int s = 0; s < K1_SPLIT_TERMS; ++s) {
            const int piece = HIDDEN_SIDE ? SPLIT_H[s] : SPLIT_W[s];
            *(uint4 *)(dst + (tile * KT + (long)s * kseg + kk) * (long)TILE_BYTES + in_block) = q[piece];
        }
    }
}

}  // namespace

hipError_t k1_pack_rows_f32_split(const void *src, int64_t rows, int d, bool hidden_side, void *dst, hipStream_t st)
{
    if (rows <= 0)
        return hipSuccess;
    const long tiles = (rows + 255) / 256;
    const int kseg = k1_split_segment(d) / BK;
    if (tiles > 0x7fffffffL || k_steps((int)k1_contraction_len(DT_F32, d)) != K1_SPLIT_TERMS * kseg)
        return hipErrorInvalidValue;
    const int rows_per_wg = tiles * ((kseg + 7) / 8) >= 1024 ? 256 : 32;
    const dim3 grid((unsigned)tiles, (kseg + 7) / 8, 256 / rows_per_wg);
    if (hidden_side)
        hipLaunchKernelGGL(pack_rows_f32_split_kernel<true>, grid, dim3(256), 0, st, (const float *)src, (long)rows,
                           d, kseg, rows_per_wg, (unsigned char *)dst);
    else
        hipLaunchKernelGGL(pack_rows_f32_split_kernel<false>, grid, dim3(256), 0, st, (const float *)src, (long)rows,
                           d, kseg, rows_per_wg, (unsigned char *)dst);
    return hipGetLastError();
}

size_t k1_packed_bytes(int64_t rows, int K)
{
    const int64_t tiles = (rows + 255) / 256;
    const int64_t kt = k_steps(K);
    return (size_t)(tiles * kt) * TILE_BYTES;
}

hipError_t k1_pack_rows_bf16(const void *src, int64_t rows, int d, void *dst, hipStream_t st)
{
    if (rows <= 0)
        return hipSuccess;
    const long tiles = (rows + 255) / 256;
    const int kt = k_steps(d);
    if (tiles > 0x7fffffffL)
        return hipErrorInvalidValue;
    // whole tiles per workgroup when there are many of them, 32-row groups when a small batch
    // would otherwise leave most of the chip idle
    const int rows_per_wg = tiles * ((kt + 7) / 8) >= 1024 ? 256 : 32;
    hipLaunchKernelGGL(pack_rows_bf16_kernel, dim3((unsigned)tiles, (kt + 7) / 8, 256 / rows_per_wg), dim3(256), 0,
                       st, (const unsigned char *)src, (long)rows, d, kt, rows_per_wg, (unsigned char *)dst);
    return hipGetLastError();
}

hipError_t k1_merge(const float *part, int nsplit, int64_t T, float *entropy, hipStream_t st)
{
    if (nsplit >= 32) {
        const long wblocks = (T + WIDE_TOKENS - 1) / WIDE_TOKENS;
        if (wblocks <= 0 || wblocks > 0x7fffffffL)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL(k1_merge_wide_kernel, dim3((unsigned)wblocks), dim3(256), 0, st, part, nsplit, (long)T,
                           entropy);
        return hipGetLastError();
    }
    const long blocks = (T + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffL)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k1_merge_kernel, dim3((unsigned)blocks), dim3(256), 0, st, part, nsplit,
                       (long)T, entropy);
    return hipGetLastError();
}

}  // namespace egtp
