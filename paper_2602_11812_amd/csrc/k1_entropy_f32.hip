// Fused LM-head contraction + streaming entropy for fp32 inputs (Eq. 2), plain fp32 FMAs.
//
// The fp32 storage type serves small, exactness-oriented workloads, so this kernel is a
// straightforward LDS-tiled contraction: a 64-token x 64-vocabulary tile per workgroup,
// 4 x 4 logits per thread, K step 16.  As in the bf16 kernel the logits are folded into
// per-token running statistics (m, S, U) as soon as a vocabulary tile is finished and are
// never stored; the same merge kernel finishes H = ln S - U ln2 / S.
#include "k1_common.h"

namespace egtp {
namespace {

constexpr int TM = 64;   // vocabulary rows per tile
constexpr int TN = 64;   // tokens per block
constexpr int TK = 16;   // K step
constexpr int PAD = 4;

__global__ __launch_bounds__(256) void k1_entropy_f32_kernel(
    const float *__restrict__ W, const float *__restrict__ Hd, long T, int d, int V, int ntb,
    int nsplit, int tps, int ntiles_v, float *__restrict__ part)
{
    __shared__ float As[TK][TM + PAD];  // As[k][vocab row]
    __shared__ float Bs[TK][TN + PAD];  // Bs[k][token]

    const int tid = threadIdx.x;
    const int tx = tid & 15;   // vocabulary group: rows tx*4 .. tx*4+3
    const int ty = tid >> 4;   // token group:      tokens ty*4 .. ty*4+3
    const int tb = blockIdx.x % ntb;
    const int sp = blockIdx.x / ntb;
    const long tok0 = (long)tb * TN;
    const int vt_begin = sp * tps;
    const int vt_end = min(ntiles_v, vt_begin + tps);

    // loader geometry: one float4 along K per thread and operand
    const int lrow = tid >> 2;        // 0..63
    const int lk = (tid & 3) * 4;     // 0,4,8,12
    long trow = tok0 + lrow;
    trow = trow < T ? trow : T - 1;   // rows past the end re-read the last token (discarded)
    const long hrow = trow * (long)d;

    Stats st[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        st[j].m = NEG_BIG;
        st[j].S = 0.f;
        st[j].U = 0.f;
    }

    for (int vt = vt_begin; vt < vt_end; ++vt) {
        const int v0 = vt * TM;
        int vrow = v0 + lrow;
        vrow = vrow < V ? vrow : V - 1;  // rows past V re-read the last row (masked below)
        const long wrow = (long)vrow * d;

        float acc[4][4];
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[i][j] = 0.f;

        for (int k0 = 0; k0 < d; k0 += TK) {
            float4 a = make_float4(0.f, 0.f, 0.f, 0.f), b = a;
            if (k0 + lk < d) {
                a = *(const float4 *)(W + wrow + k0 + lk);
                b = *(const float4 *)(Hd + hrow + k0 + lk);
            }
            __syncthreads();  // previous step's readers are done
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

        // fold this tile's 4 logits per token into the running statistics
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            float z[4];
#pragma unroll
            for (int i = 0; i < 4; ++i)
                z[i] = (v0 + tx * 4 + i < V) ? acc[i][j] : NEG_BIG;
            const float mx = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
            if (!(mx > NEG_BIG))
                continue;  // all four rows are past the vocabulary: nothing to add
            if (mx > st[j].m) {
                const float dl = (st[j].m - mx) * LOG2E;
                const float sc = __builtin_amdgcn_exp2f(dl);
                st[j].U = (st[j].U + dl * st[j].S) * sc;
                st[j].S *= sc;
                st[j].m = mx;
            }
            const float mc = -st[j].m * LOG2E;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float t = fmaf(z[i], LOG2E, mc);
                const float e = __builtin_amdgcn_exp2f(t);
                st[j].S += e;
                st[j].U = fmaf(e, t, st[j].U);
            }
        }
    }

    // the 16 threads tx = 0..15 of a token group are 16 consecutive lanes
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int off = 1; off < 16; off <<= 1) {
            Stats o;
            o.m = __shfl_xor(st[j].m, off);
            o.S = __shfl_xor(st[j].S, off);
            o.U = __shfl_xor(st[j].U, off);
            st[j] = merge(st[j], o);
        }
    }
    if (tx == 0) {
        const long plane = (long)nsplit * T;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const long tok = tok0 + ty * 4 + j;
            if (tok < T) {
                const long idx = (long)sp * T + tok;
                part[idx] = st[j].m;
                part[plane + idx] = st[j].S;
                part[2 * plane + idx] = st[j].U;
            }
        }
    }
}

}  // namespace

hipError_t k1_entropy_f32(const void *hidden, const void *w_lm, int64_t T, int d, int V,
                          const K1Plan &p, float *part, hipStream_t st)
{
    if (p.tb_tokens != TN || p.tile_v != TM || T <= 0)
        return hipErrorInvalidValue;
    const long units = (long)p.ntb * p.nsplit;
    if (units <= 0 || units > 0x7fffffffL)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k1_entropy_f32_kernel, dim3((unsigned)units), dim3(256), 0, st, (const float *)w_lm,
                       (const float *)hidden, (long)T, d, V, p.ntb, p.nsplit, p.tiles_per_split, p.ntiles_v,
                       part);
    return hipGetLastError();
}

}  // namespace egtp
