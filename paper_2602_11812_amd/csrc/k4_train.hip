// One optimisation step of a K-bin prediction head on frozen features (Section 3.2, 3.3):
// soft labels of Eq. 5, the joint loss of Eq. 7, the per-sequence step average of Eq. 9
// (as a per-sample weight), the backward pass through the head only, and AdamW.
//
// Everything is fp32 (master weights, moments, activations).  Three launches:
//   1. layer 1 forward     partial pre-activations, split along d   (shared with scoring)
//   2. per-sample kernel   ReLU, logits, softmax, expected value, soft label, the two loss
//                          terms, d loss / d logits and d loss / d pre-activation
//   3. the updates, one grid of three kinds of workgroups that only need what 2. left behind:
//      W1                  gradient tile [64 x 64] of  dact^T . x  accumulated over the batch in
//                          registers and consumed by AdamW on the spot -- the d_h x d gradient
//                          is never written unless the caller asks for a copy.  With the
//                          paper's batch of 16 this part is a pure stream over W1 and its two
//                          moments (read and written once each).
//      small parameters    gradient of W2, b2 and b1 reduced over the batch in a fixed order,
//                          AdamW applied in the same thread
//      loss                fixed-order sum of the per-sample terms (the last workgroup)
// No floating-point atomics anywhere: results are bit-reproducible.
#include "kernels.h"
#include "partial_planes.h"
#include "wave_reduce.h"

namespace egtp {
namespace {

struct Adam {
    float lr, beta1, beta2, omb1, omb2, eps, wd, corr1, corr2;
};

// decoupled weight decay: w <- w - lr wd w - lr mhat / (sqrt(vhat) + eps)
__device__ __forceinline__ void adamw(const Adam &h, float g, float &w, float &m, float &v)
{
    m = h.beta1 * m + h.omb1 * g;
    v = h.beta2 * v + h.omb2 * g * g;
    const float mhat = m / h.corr1;
    const float vhat = v / h.corr2;
    w = w - h.lr * h.wd * w - h.lr * mhat / (sqrtf(vhat) + h.eps);
}

// ---- 2. one workgroup per sample ---------------------------------------------------------
// LDS: a[d_h] | z[K] | dz[K]
__global__ __launch_bounds__(256) void train_sample_kernel(
    const float *__restrict__ act_part, int nks, int B, int d_h, int K, const float *__restrict__ b1,
    const float *__restrict__ w2, const float *__restrict__ b2, const float *__restrict__ centers,
    const int32_t *__restrict__ bin, const float *__restrict__ y, const int32_t *__restrict__ steps, int n_seqs,
    float lambda, float *__restrict__ act, float *__restrict__ dact, float *__restrict__ dz_out,
    float *__restrict__ loss_part)
{
    extern __shared__ __align__(16) float sm[];
    float *a = sm;
    float *z = a + d_h;
    float *dz = z + K;
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    // pre-activations: the slices' partial sums, added in slice order
    if ((d_h & 3) == 0) {
        for (int j = tid * 4; j < d_h; j += 1024) {
            const float4 pre = sum_planes4(act_part, nks, B, b, d_h, j);
            float4 r;  // the caller's bias vector need not be 16-byte aligned
            r.x = fmaxf(pre.x + b1[j], 0.f), r.y = fmaxf(pre.y + b1[j + 1], 0.f);
            r.z = fmaxf(pre.z + b1[j + 2], 0.f), r.w = fmaxf(pre.w + b1[j + 3], 0.f);
            *(float4 *)(a + j) = r;
            *(float4 *)(act + (long)b * d_h + j) = r;
        }
    } else {
        for (int j = tid; j < d_h; j += 256) {
            float pre = 0.f;
#pragma unroll 8
            for (int s = 0; s < nks; ++s)
                pre += act_part[((long)s * B + b) * d_h + j];
            pre += b1[j];
            const float r = pre > 0.f ? pre : 0.f;
            a[j] = r;
            act[(long)b * d_h + j] = r;
        }
    }
    __syncthreads();
    // logits: a wave takes OUTS_AT_ONCE outputs at a time so that their weight loads are all in flight together
    // (W2 is small and cache-resident; what costs is the latency of each dependent round of loads)
    constexpr int OUTS_AT_ONCE = 5;
    for (int o0 = wave * OUTS_AT_ONCE; o0 < K; o0 += 4 * OUTS_AT_ONCE) {
        float s[OUTS_AT_ONCE];
#pragma unroll
        for (int q = 0; q < OUTS_AT_ONCE; ++q)
            s[q] = 0.f;
#pragma unroll 4
        for (int j = lane; j < d_h; j += 64) {
            const float aj = a[j];
#pragma unroll
            for (int q = 0; q < OUTS_AT_ONCE; ++q) {
                const int o = o0 + q < K ? o0 + q : K - 1;  // past the end: a valid row, not used
                s[q] = fmaf(w2[(long)o * d_h + j], aj, s[q]);
            }
        }
#pragma unroll
        for (int q = 0; q < OUTS_AT_ONCE; ++q) {
            const float t = wave_sum(s[q]);
            if (lane == 0 && o0 + q < K)
                z[o0 + q] = t + b2[o0 + q];
        }
    }
    __syncthreads();
    if (wave == 0) {
        int i = bin[b];
        i = i < 0 ? 0 : (i >= K ? K - 1 : i);
        float m = -__builtin_inff();
        for (int o = lane; o < K; o += 64)
            m = fmaxf(m, z[o]);
        m = wave_max(m);
        float S = 0.f, Zl = 0.f;  // normalisers of the prediction and of the soft label (Eq. 5)
        for (int o = lane; o < K; o += 64) {
            S += expf(z[o] - m);
            Zl += expf(-fabsf((float)(o - i)));
        }
        S = wave_sum(S);
        Zl = wave_sum(Zl);
        const float lnS = logf(S);
        float yhat = 0.f, ce = 0.f;
        for (int o = lane; o < K; o += 64) {
            const float ph = expf(z[o] - m) / S;
            const float p = expf(-fabsf((float)(o - i))) / Zl;
            yhat = fmaf(ph, centers[o], yhat);  // Eq. 6
            ce -= p * ((z[o] - m) - lnS);
        }
        yhat = wave_sum(yhat);
        ce = wave_sum(ce);
        const float err = yhat - y[b];
        // Eq. 9: a sequence's steps share its 1/N; without step counts every sample weighs 1/B
        const float wb = steps ? 1.0f / ((float)n_seqs * (float)steps[b]) : 1.0f / (float)B;
        for (int o = lane; o < K; o += 64) {
            const float ph = expf(z[o] - m) / S;
            const float p = expf(-fabsf((float)(o - i))) / Zl;
            const float g = wb * (lambda * (ph - p) + (1.0f - lambda) * 2.0f * err * ph * (centers[o] - yhat));
            dz[o] = g;
            dz_out[(long)b * K + o] = g;
        }
        if (lane == 0) {
            loss_part[2 * b] = wb * ce;
            loss_part[2 * b + 1] = wb * err * err;
        }
    }
    __syncthreads();
    // d loss / d pre-activation = (W2^T dz) where the unit is active; many rows of W2 in flight per thread
    for (int j = tid; j < d_h; j += 256) {
        float s = 0.f;
#pragma unroll 20
        for (int o = 0; o < K; ++o)
            s = fmaf(dz[o], w2[(long)o * d_h + j], s);
        dact[(long)b * d_h + j] = a[j] > 0.f ? s : 0.f;
    }
}

// ---- 5. loss = {lambda CE + (1 - lambda) MSE, CE, MSE}, fixed summation order -----------------
// (one workgroup of 256 threads; runs as the last workgroup of the update launch)
__device__ void sum_loss(const float *__restrict__ loss_part, int B, float lambda, float *__restrict__ loss)
{
    __shared__ float red[2][256];
    const int tid = threadIdx.x;
    float ce = 0.f, mse = 0.f;
    for (int b = tid; b < B; b += 256) {
        ce += loss_part[2 * b];
        mse += loss_part[2 * b + 1];
    }
    red[0][tid] = ce;
    red[1][tid] = mse;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if (tid < s) {
            red[0][tid] += red[0][tid + s];
            red[1][tid] += red[1][tid + s];
        }
        __syncthreads();
    }
    if (tid == 0) {
        loss[0] = lambda * red[0][0] + (1.0f - lambda) * red[1][0];
        loss[1] = red[0][0];
        loss[2] = red[1][0];
    }
}

// ---- 3. W2, b2, b1: one thread per parameter (workgroup `block` of the small-parameter part) ----
__device__ __forceinline__ void small_update(
    int block, const float *__restrict__ act, const float *__restrict__ dact, const float *__restrict__ dz, int B,
    int d_h, int K, const Adam &h, float *__restrict__ w2, float *__restrict__ m_w2, float *__restrict__ v_w2,
    float *__restrict__ b2, float *__restrict__ m_b2, float *__restrict__ v_b2, float *__restrict__ b1,
    float *__restrict__ m_b1, float *__restrict__ v_b1, float *__restrict__ g_w2, float *__restrict__ g_b2,
    float *__restrict__ g_b1)
{
    const long e = (long)block * 256 + threadIdx.x;
    const long n_w2 = (long)K * d_h;
    float g = 0.f;
    float *w, *m, *v, *gout;
    if (e < n_w2) {
        const int o = (int)(e / d_h), j = (int)(e - (long)o * d_h);
        for (int b = 0; b < B; ++b)
            g = fmaf(dz[(long)b * K + o], act[(long)b * d_h + j], g);
        w = w2 + e, m = m_w2 + e, v = v_w2 + e, gout = g_w2 ? g_w2 + e : nullptr;
    } else if (e < n_w2 + K) {
        const int o = (int)(e - n_w2);
        for (int b = 0; b < B; ++b)
            g += dz[(long)b * K + o];
        w = b2 + o, m = m_b2 + o, v = v_b2 + o, gout = g_b2 ? g_b2 + o : nullptr;
    } else if (e < n_w2 + K + d_h) {
        const int j = (int)(e - n_w2 - K);
        for (int b = 0; b < B; ++b)
            g += dact[(long)b * d_h + j];
        w = b1 + j, m = m_b1 + j, v = v_b1 + j, gout = g_b1 ? g_b1 + j : nullptr;
    } else {
        return;
    }
    float wv = *w, mv = *m, vv = *v;
    adamw(h, g, wv, mv, vv);
    *w = wv;
    *m = mv;
    *v = vv;
    if (gout)
        *gout = g;
}

// ---- 4. W1: gradient tile in registers, AdamW in the epilogue -------------------------------
constexpr int GM = 64;  // rows j of W1 per tile
constexpr int GN = 64;  // columns k of W1 per tile
constexpr int GB = 16;  // samples per LDS stage

__device__ __forceinline__ void w1_update(
    int tile_k, int tile_j, const float *__restrict__ x, const float *__restrict__ dact, int B, int d, int d_h,
    const Adam &h, float *__restrict__ w1, float *__restrict__ m_w1, float *__restrict__ v_w1,
    float *__restrict__ g_w1)
{
    __shared__ __align__(16) float As[GB][GM];  // dact[b][j]
    __shared__ __align__(16) float Bs[GB][GN];  // x[b][k]
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int k0 = tile_k * GN, j0 = tile_j * GM;
    const int lb = tid >> 4;        // sample row this thread stages
    const int lc = (tid & 15) * 4;  // first of its four columns

    float acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int c = 0; c < 4; ++c)
            acc[i][c] = 0.f;

    for (int b0 = 0; b0 < B; b0 += GB) {
        float4 av = make_float4(0.f, 0.f, 0.f, 0.f), bv = av;
        const int b = b0 + lb;
        if (b < B) {
            const float *dp = dact + (long)b * d_h + j0 + lc;
            av.x = j0 + lc + 0 < d_h ? dp[0] : 0.f;
            av.y = j0 + lc + 1 < d_h ? dp[1] : 0.f;
            av.z = j0 + lc + 2 < d_h ? dp[2] : 0.f;
            av.w = j0 + lc + 3 < d_h ? dp[3] : 0.f;
            if (k0 + lc < d)  // d is a multiple of 4: the whole quad is inside the row
                bv = *(const float4 *)(x + (long)b * d + k0 + lc);
        }
        __syncthreads();
        *(float4 *)&As[lb][lc] = av;
        *(float4 *)&Bs[lb][lc] = bv;
        __syncthreads();
#pragma unroll
        for (int bb = 0; bb < GB; ++bb) {
            const float4 a4 = *(const float4 *)&As[bb][ty * 4];
            const float4 b4 = *(const float4 *)&Bs[bb][tx * 4];
            const float aa[4] = {a4.x, a4.y, a4.z, a4.w};
            const float kk[4] = {b4.x, b4.y, b4.z, b4.w};
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int c = 0; c < 4; ++c)
                    acc[i][c] = fmaf(aa[i], kk[c], acc[i][c]);
        }
    }
    const int k = k0 + tx * 4;
    if (k >= d)
        return;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int j = j0 + ty * 4 + i;
        if (j >= d_h)
            continue;
        const long at = (long)j * d + k;
        float4 w = *(const float4 *)(w1 + at);
        float4 m = *(const float4 *)(m_w1 + at);
        float4 v = *(const float4 *)(v_w1 + at);
        adamw(h, acc[i][0], w.x, m.x, v.x);
        adamw(h, acc[i][1], w.y, m.y, v.y);
        adamw(h, acc[i][2], w.z, m.z, v.z);
        adamw(h, acc[i][3], w.w, m.w, v.w);
        *(float4 *)(w1 + at) = w;
        *(float4 *)(m_w1 + at) = m;
        *(float4 *)(v_w1 + at) = v;
        if (g_w1)
            *(float4 *)(g_w1 + at) = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    }
}

// ---- 3. + 4. + 5. in one launch: all three need only what the per-sample kernel left behind and touch
// disjoint parameters, so they share a grid.  The W1 tiles come first in launch order (they carry the
// memory traffic of the step), then the workgroups of the small parameters, the loss last.
struct UpdateArgs {
    const float *x, *act, *dact, *dz, *loss_part;
    int B, d, d_h, K;
    int tiles_k, tiles_w1, blocks_small;
    float lambda;
    float *w1, *m_w1, *v_w1, *g_w1;
    float *w2, *m_w2, *v_w2, *g_w2;
    float *b2, *m_b2, *v_b2, *g_b2;
    float *b1, *m_b1, *v_b1, *g_b1;
    float *loss;
};

__global__ __launch_bounds__(256) void train_update_kernel(UpdateArgs a, Adam h)
{
    const int id = blockIdx.x;
    if (id < a.tiles_w1) {
        w1_update(id % a.tiles_k, id / a.tiles_k, a.x, a.dact, a.B, a.d, a.d_h, h, a.w1, a.m_w1, a.v_w1, a.g_w1);
    } else if (id < a.tiles_w1 + a.blocks_small) {
        small_update(id - a.tiles_w1, a.act, a.dact, a.dz, a.B, a.d_h, a.K, h, a.w2, a.m_w2, a.v_w2, a.b2, a.m_b2,
                     a.v_b2, a.b1, a.m_b1, a.v_b1, a.g_w2, a.g_b2, a.g_b1);
    } else {
        sum_loss(a.loss_part, a.B, a.lambda, a.loss);
    }
}

}  // namespace

hipError_t head_train_step(const TrainArgs &a, hipStream_t st)
{
    if (a.B <= 0)
        return hipSuccess;
    if (a.d % 4 != 0)
        return hipErrorInvalidValue;
    const size_t lds = ((size_t)a.d_h + 2 * (size_t)a.K) * sizeof(float);
    if (lds > 96 * 1024)
        return hipErrorInvalidValue;
    static DeviceMask lds_limit_raised{0};
    hipError_t ea = raise_dynamic_lds_limit((const void *)train_sample_kernel, 96 * 1024, lds_limit_raised);
    if (ea != hipSuccess)
        return ea;
    hipError_t e = head_layer1(a.x, nullptr, a.B, a.d, a.d_h, a.w1, DT_F32, a.act_part, st);
    if (e != hipSuccess)
        return e;
    hipLaunchKernelGGL(train_sample_kernel, dim3(a.B), dim3(256), lds, st, a.act_part, head_k_splits(a.d, a.d_h, a.B, DT_F32), a.B,
                       a.d_h, a.K, a.b1, a.w2, a.b2, a.centers, a.bin, a.y, a.steps, a.n_seqs, a.lambda, a.act,
                       a.dact, a.dz, a.loss_part);
    Adam h;
    h.lr = a.lr;
    h.beta1 = a.beta1;
    h.beta2 = a.beta2;
    h.omb1 = a.omb1;
    h.omb2 = a.omb2;
    h.eps = a.eps;
    h.wd = a.weight_decay;
    h.corr1 = a.corr1;
    h.corr2 = a.corr2;
    // the parameter updates come last: the forward and the backward pass above read the old W1 / W2
    UpdateArgs u;
    u.x = a.x, u.act = a.act, u.dact = a.dact, u.dz = a.dz, u.loss_part = a.loss_part;
    u.B = a.B, u.d = a.d, u.d_h = a.d_h, u.K = a.K;
    u.lambda = a.lambda;
    u.w1 = a.w1, u.m_w1 = a.m_w1, u.v_w1 = a.v_w1, u.g_w1 = a.g_w1;
    u.w2 = a.w2, u.m_w2 = a.m_w2, u.v_w2 = a.v_w2, u.g_w2 = a.g_w2;
    u.b2 = a.b2, u.m_b2 = a.m_b2, u.v_b2 = a.v_b2, u.g_b2 = a.g_b2;
    u.b1 = a.b1, u.m_b1 = a.m_b1, u.v_b1 = a.v_b1, u.g_b1 = a.g_b1;
    u.loss = a.loss;
    const long n_small = (long)a.K * a.d_h + a.K + a.d_h;
    const long tiles_k = (a.d + GN - 1) / GN, tiles_j = (a.d_h + GM - 1) / GM;
    const long blocks_small = (n_small + 255) / 256;
    if (tiles_k * tiles_j + blocks_small + 1 > 0x7fffffffL)
        return hipErrorInvalidValue;
    u.tiles_k = (int)tiles_k;
    u.tiles_w1 = (int)(tiles_k * tiles_j);
    u.blocks_small = (int)blocks_small;
    hipLaunchKernelGGL(train_update_kernel, dim3((unsigned)(u.tiles_w1 + u.blocks_small + 1)), dim3(256), 0, st, u, h);
    return hipGetLastError();
}

}  // namespace egtp
