// Entropy-softmax weights and weighted pooling over ragged offsets (Eq. 3, Eq. 4), the
// streaming PLP fold of Eq. 8, the ablation poolers of Table 3, and the ragged plumbing.
//
// Pooling is HBM-bound: every hidden state is read once more (16 bytes per lane, a wave
// reads 1 KiB of one token row at a time).  A sequence is cut into units of at most
// POOL_UNIT tokens so that long and short sequences load the chip evenly; each unit leaves a
// partial weighted sum (already normalised with the sequence's final log-sum-exp), and a
// finalize kernel adds a sequence's partials in unit order.  No atomics: bit-reproducible.
#include "k1_common.h"
#include "stream_load.h"
#include "wave_reduce.h"

namespace egtp {
namespace {

constexpr float NEG_INF = -__builtin_inff();

// ---- block reductions (256 threads), fixed tree => deterministic ---------------------
__device__ float block_max(float v, float *sh)
{
    v = wave_max(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
        sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return fmaxf(fmaxf(sh[0], sh[1]), fmaxf(sh[2], sh[3]));
}
__device__ float block_sum(float v, float *sh)
{
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0)
        sh[threadIdx.x >> 6] = v;
    __syncthreads();
    return (sh[0] + sh[1]) + (sh[2] + sh[3]);
}

// ---- ragged plumbing ---------------------------------------------------------------------
// offsets[0..B] = exclusive scan of f(lengths[b]); one workgroup walks the array in chunks
// of 256 with a running carry.  UNITS: scan ceil(n_b / POOL_UNIT) of n_b = in[b+1]-in[b].
template <bool UNITS>
__global__ __launch_bounds__(256) void scan_kernel(const int32_t *__restrict__ in, int32_t B,
                                                   int32_t *__restrict__ out)
{
    __shared__ int sh[256];
    __shared__ int carry;
    const int tid = threadIdx.x;
    if (tid == 0) {
        carry = 0;
        out[0] = 0;
    }
    __syncthreads();
    for (int base = 0; base < B; base += 256) {
        const int b = base + tid;
        int v = 0;
        if (b < B) {
            if (UNITS) {
                const int n = in[b + 1] - in[b];
                v = n > 0 ? (n + POOL_UNIT - 1) / POOL_UNIT : 0;
            } else {
                v = in[b];
            }
        }
        sh[tid] = v;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {  // inclusive Hillis-Steele scan
            int add = tid >= o ? sh[tid - o] : 0;
            __syncthreads();
            sh[tid] += add;
            __syncthreads();
        }
        if (b < B)
            out[b + 1] = carry + sh[tid];
        __syncthreads();
        if (tid == 255)
            carry += sh[255];
        __syncthreads();
    }
}

// largest b in [0, B) with arr[b] <= t, given arr[0] <= t < arr[B], arr non-decreasing
__device__ __forceinline__ int find_segment(const int32_t *__restrict__ arr, int B, long t)
{
    int lo = 0, hi = B;  // invariant: arr[lo] <= t < arr[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (arr[mid] <= t)
            lo = mid;
        else
            hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(256) void seg_ids_kernel(const int32_t *__restrict__ offsets, int32_t B,
                                                      long T, int32_t *__restrict__ seg)
{
    const long t = (long)blockIdx.x * 256 + threadIdx.x;
    if (t >= T)
        return;
    seg[t] = (B > 0 && t < offsets[B]) ? find_segment(offsets, B, t) : -1;
}

// Device offsets are the caller's: whatever they hold, no token index leaves [0, T] and no unit
// index leaves the partial buffer (a malformed table gives wrong numbers, not wild accesses).
__device__ __forceinline__ long clamp_token(long t, long T) { return t < 0 ? 0 : (t > T ? T : t); }

// ---- Eq. 3: per-sequence log-sum-exp of H/alpha, joined with the old state's lse ---------
__global__ __launch_bounds__(256) void pool_lse_kernel(const float *__restrict__ entropy,
                                                       const int32_t *__restrict__ offsets, long T,
                                                       const int32_t *__restrict__ slot, float inv_alpha,
                                                       const float *__restrict__ state_lse,
                                                       float *__restrict__ lse_new,
                                                       float *__restrict__ state_scale)
{
    __shared__ float sh[4];
    const int b = blockIdx.x;
    const int lo = (int)clamp_token(offsets[b], T), hi = (int)clamp_token(offsets[b + 1], T);
    const int s = slot ? slot[b] : b;
    const float L_old = state_lse ? state_lse[s] : NEG_INF;
    float mx = NEG_INF;
    for (int i = lo + threadIdx.x; i < hi; i += 256)
        mx = fmaxf(mx, entropy[i] * inv_alpha);
    mx = fmaxf(block_max(mx, sh), L_old);
    float sum = 0.f;
    if (mx > NEG_INF)
        for (int i = lo + threadIdx.x; i < hi; i += 256)
            sum += __expf(entropy[i] * inv_alpha - mx);
    sum = block_sum(sum, sh);
    if (threadIdx.x == 0) {
        float L = NEG_INF, sc = 0.f;
        if (mx > NEG_INF) {
            const float old = L_old > NEG_INF ? __expf(L_old - mx) : 0.f;
            L = mx + __logf(sum + old);
            sc = L_old > NEG_INF ? __expf(L_old - L) : 0.f;
        }
        lse_new[b] = L;
        state_scale[b] = sc;
    }
}

// ---- Eq. 4: partial weighted sums per unit --------------------------------------------------
// MODE 0: weights e^{H/alpha - lse} (Eq. 3-4); MODE 1: plain sums (average pooling, divided by the
// length when the units are joined); MODE 2: element-wise maxima.
enum : int { POOL_WEIGHTED = 0, POOL_SUM = 1, POOL_MAXIMUM = 2 };

template <bool BF16, typename Q>
__device__ __forceinline__ void widen16(const Q &q, float (&h)[BF16 ? 8 : 4])
{
    if (BF16) {
        const unsigned v[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            h[2 * e] = __uint_as_float(v[e] << 16);
            h[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
        }
    } else {
        h[0] = __uint_as_float(q.x);
        h[1] = __uint_as_float(q.y);
        h[2] = __uint_as_float(q.z);
        h[3] = __uint_as_float(q.w);
    }
}

template <bool BF16, int MODE>
__global__ __launch_bounds__(256) void pool_partial_kernel(
    const void *__restrict__ hidden, int d, const float *__restrict__ entropy,
    const int32_t *__restrict__ offsets, int32_t B, long T, float inv_alpha, const float *__restrict__ lse_new,
    const int32_t *__restrict__ unit_start, int ysplit, float *__restrict__ partial)
{
    __shared__ float w[POOL_UNIT];
    // Workgroup = (unit, feature slice), the slice varying fastest so that the slices of a unit -- pieces of
    // the same token rows -- are read at about the same time.  The grid holds pool_units_bound(T, B) units:
    // u indexes inside the partial buffer.
    const int u = blockIdx.x / ysplit;
    const int yslice = blockIdx.x - u * ysplit;
    if (u >= unit_start[B])
        return;
    const int b = find_segment(unit_start, B, u);
    const long t0 = clamp_token((long)offsets[b] + (long)(u - unit_start[b]) * POOL_UNIT, T);
    const int n = (int)max(0L, min((long)POOL_UNIT, clamp_token(offsets[b + 1], T) - t0));
    if (MODE == POOL_WEIGHTED) {
        if (threadIdx.x < POOL_UNIT)
            w[threadIdx.x] = threadIdx.x < n ? __expf(entropy[t0 + threadIdx.x] * inv_alpha - lse_new[b]) : 0.f;
        __syncthreads();
    }

    constexpr int VEC = BF16 ? 8 : 4;  // elements per 16-byte load
    const int nchunk = d / VEC;
    float *out = partial + (long)u * d;
    // a slice is 256 chunks of 16 bytes, one per thread (two slices at d = 4096: twice as many workgroups as
    // units, which evens out the end of the launch)
    for (int c = yslice * 256 + threadIdx.x; c < nchunk; c += 256 * ysplit) {
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e)
            acc[e] = MODE == POOL_MAXIMUM ? NEG_INF : 0.f;
        const unsigned char *p = (const unsigned char *)hidden + (t0 * d + (long)c * VEC) * (BF16 ? 2 : 4);
        const long stride = (long)d * (BF16 ? 2 : 4);
        auto fold = [&](const u32x4 &q, int i) {
            float h[VEC];
            widen16<BF16>(q, h);
            const float wi = MODE == POOL_WEIGHTED ? w[i] : 1.f;
#pragma unroll
            for (int e = 0; e < VEC; ++e)
                acc[e] = MODE == POOL_MAXIMUM ? fmaxf(acc[e], h[e])
                         : MODE == POOL_SUM   ? acc[e] + h[e]
                                              : fmaf(wi, h[e], acc[e]);
        };
        int i = 0;
        for (; i + 8 <= n; i += 8) {  // eight rows in flight per thread
            u32x4 q[8];
#pragma unroll
            for (int r = 0; r < 8; ++r)
                q[r] = stream_load16(p + (long)(i + r) * stride);
#pragma unroll
            for (int r = 0; r < 8; ++r)
                fold(q[r], i + r);
        }
        for (; i < n; ++i)
            fold(stream_load16(p + (long)i * stride), i);
#pragma unroll
        for (int e = 0; e < VEC; e += 4)
            *(float4 *)(out + (long)c * VEC + e) = make_float4(acc[e], acc[e + 1], acc[e + 2], acc[e + 3]);
    }
}

// ---- joining a sequence's unit partials ----------------------------------------------------------
// Thread = four consecutive features of one sequence; the partials are combined in unit order (a fixed
// order: bit-reproducible), JOIN_AHEAD of them fetched before any is used -- a sequence of 8192 tokens
// has 64 units, and one load at a time would make the join a chain of 64 memory latencies.
constexpr int JOIN_AHEAD = 8;

template <int MODE>
__device__ __forceinline__ float4 join_units(const float *__restrict__ partial, int u0, int u1, int d, int k,
                                             float init)
{
    float4 r = make_float4(init, init, init, init);
    auto add = [&](const float4 &v) {
        if (MODE == POOL_MAXIMUM) {
            r.x = fmaxf(r.x, v.x), r.y = fmaxf(r.y, v.y), r.z = fmaxf(r.z, v.z), r.w = fmaxf(r.w, v.w);
        } else {
            r.x += v.x, r.y += v.y, r.z += v.z, r.w += v.w;
        }
    };
    int u = u0;
    for (; u + JOIN_AHEAD <= u1; u += JOIN_AHEAD) {
        float4 v[JOIN_AHEAD];
#pragma unroll
        for (int i = 0; i < JOIN_AHEAD; ++i)
            v[i] = *(const float4 *)(partial + (long)(u + i) * d + k);
#pragma unroll
        for (int i = 0; i < JOIN_AHEAD; ++i)
            add(v[i]);
    }
    for (; u < u1; ++u)
        add(*(const float4 *)(partial + (long)u * d + k));
    return r;
}

// Table 3 alternatives: sum / length, or maximum
template <int MODE>
__global__ __launch_bounds__(256) void pool_finalize_plain_kernel(const float *__restrict__ partial,
                                                                  const int32_t *__restrict__ unit_start,
                                                                  const int32_t *__restrict__ offsets, int d,
                                                                  int units_cap, float *__restrict__ out_pooled)
{
    const int b = blockIdx.x;
    const int k = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (k >= d)
        return;
    const int u0 = unit_start[b], u1 = min(unit_start[b + 1], units_cap);
    const int len = offsets[b + 1] - offsets[b];
    // an empty sequence pools to zero
    float4 r = join_units<MODE>(partial, u0, u1, d, k, (MODE == POOL_MAXIMUM && len > 0) ? NEG_INF : 0.f);
    if (MODE == POOL_SUM && len > 0) {
        const float inv = 1.0f / (float)len;
        r.x *= inv, r.y *= inv, r.z *= inv, r.w *= inv;
    }
    *(float4 *)(out_pooled + (long)b * d + k) = r;
}

// Eq. 4 / Eq. 8: the sum of a sequence's partials plus the rescaled old state
__global__ __launch_bounds__(256) void pool_finalize_kernel(
    const float *__restrict__ partial, const int32_t *__restrict__ unit_start,
    const int32_t *__restrict__ slot, int d, int units_cap, const float *state_pooled,
    const float *__restrict__ state_scale, const float *__restrict__ lse_new, float *out_pooled,
    float *out_lse)
{
    const int b = blockIdx.x;
    const int k = (blockIdx.y * 256 + threadIdx.x) * 4;
    const int s = slot ? slot[b] : b;
    if (k < d) {
        const int u0 = unit_start[b], u1 = min(unit_start[b + 1], units_cap);
        float4 sum = join_units<POOL_SUM>(partial, u0, u1, d, k, 0.f);
        const float sc = state_scale[b];
        if (state_pooled && sc != 0.f) {
            const float4 old = *(const float4 *)(state_pooled + (long)s * d + k);
            sum.x = fmaf(old.x, sc, sum.x), sum.y = fmaf(old.y, sc, sum.y);
            sum.z = fmaf(old.z, sc, sum.z), sum.w = fmaf(old.w, sc, sum.w);
        }
        *(float4 *)(out_pooled + (long)s * d + k) = sum;
    }
    if (blockIdx.y == 0 && threadIdx.x == 0)
        out_lse[s] = lse_new[b];
}

// ---- Eq. 8 fast path: exactly one new token per sequence ------------------------------------
// With part != NULL the kernel first finishes Eq. 2 for its token -- the nsplit partial (m, S, U) triples the
// fused kernel left for it are merged by a fixed tree (thread i takes ranges i, i + 256, ... in order, then an
// xor tree inside each wave, then the four waves in order) -- and writes H to entropy[b]; otherwise entropy[b]
// is read.
template <bool BF16>
__global__ __launch_bounds__(256) void plp_fold1_kernel(const void *__restrict__ hidden, int d, float *entropy,
                                                        const float *__restrict__ part, int nsplit, long T,
                                                        const int32_t *__restrict__ slot, float inv_alpha,
                                                        float *pooled_state, float *lse_state)
{
    __shared__ float red[4][3];
    const int b = blockIdx.x;
    const int s = slot ? slot[b] : b;
    float H;
    if (part != nullptr) {
        const long plane = (long)nsplit * T;
        Stats acc;
        acc.m = NEG_BIG, acc.S = 0.f, acc.U = 0.f;
        for (int r = threadIdx.x; r < nsplit; r += 256) {
            const long idx = (long)r * T + b;
            Stats o;
            o.m = part[idx], o.S = part[plane + idx], o.U = part[2 * plane + idx];
            acc = merge(acc, o);
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            Stats o;
            o.m = __shfl_xor(acc.m, off), o.S = __shfl_xor(acc.S, off), o.U = __shfl_xor(acc.U, off);
            acc = merge(acc, o);
        }
        if ((threadIdx.x & 63) == 0) {
            red[threadIdx.x >> 6][0] = acc.m;
            red[threadIdx.x >> 6][1] = acc.S;
            red[threadIdx.x >> 6][2] = acc.U;
        }
        __syncthreads();
        acc.m = red[0][0], acc.S = red[0][1], acc.U = red[0][2];
#pragma unroll
        for (int k = 1; k < 4; ++k) {
            Stats o;
            o.m = red[k][0], o.S = red[k][1], o.U = red[k][2];
            acc = merge(acc, o);
        }
        H = logf(acc.S) - acc.U * 0.6931471805599453f / acc.S;
        if (threadIdx.x == 0)
            entropy[b] = H;
    } else {
        H = entropy[b];
    }
    const float L_old = lse_state[s];
    const float a = H * inv_alpha;
    const float M = fmaxf(L_old, a);
    const float old = L_old > NEG_INF ? __expf(L_old - M) : 0.f;
    const float L = M + __logf(old + __expf(a - M));
    const float sc = L_old > NEG_INF ? __expf(L_old - L) : 0.f;
    const float wn = __expf(a - L);
    __syncthreads();  // every thread has read the old lse before it is replaced
    if (threadIdx.x == 0)
        lse_state[s] = L;

    constexpr int VEC = BF16 ? 8 : 4;
    const int nchunk = d / VEC;
    const unsigned char *hp = (const unsigned char *)hidden + (long)b * d * (BF16 ? 2 : 4);
    float *pp = pooled_state + (long)s * d;
    for (int c = threadIdx.x; c < nchunk; c += 256) {
        const uint4 q = *(const uint4 *)(hp + (long)c * 16);
        float h[VEC];
        if (BF16) {
            const unsigned v[4] = {q.x, q.y, q.z, q.w};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                h[2 * e] = __uint_as_float(v[e] << 16);
                h[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
            }
        } else {
            h[0] = __uint_as_float(q.x);
            h[1] = __uint_as_float(q.y);
            h[2] = __uint_as_float(q.z);
            h[3] = __uint_as_float(q.w);
        }
#pragma unroll
        for (int e = 0; e < VEC; e += 4) {
            float4 p = make_float4(0.f, 0.f, 0.f, 0.f);
            if (sc != 0.f)
                p = *(const float4 *)(pp + (long)c * VEC + e);
            p.x = fmaf(p.x, sc, wn * h[e]);
            p.y = fmaf(p.y, sc, wn * h[e + 1]);
            p.z = fmaf(p.z, sc, wn * h[e + 2]);
            p.w = fmaf(p.w, sc, wn * h[e + 3]);
            *(float4 *)(pp + (long)c * VEC + e) = p;
        }
    }
}

// ---- Table 3 alternative: the last token's hidden state ------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void pool_last_kernel(const void *__restrict__ hidden, int d,
                                                        const int32_t *__restrict__ offsets, long T,
                                                        float *__restrict__ out_pooled)
{
    constexpr int VEC = BF16 ? 8 : 4;
    const int b = blockIdx.x;
    const int c = blockIdx.y * 256 + threadIdx.x;
    if (c * VEC >= d)
        return;
    const long lo = clamp_token(offsets[b], T), hi = clamp_token(offsets[b + 1], T);
    float h[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        h[e] = 0.f;  // an empty sequence pools to zero
    if (hi > lo) {
        const uint4 q = *(const uint4 *)((const unsigned char *)hidden + ((hi - 1) * d + (long)c * VEC) * (BF16 ? 2 : 4));
        widen16<BF16>(q, h);
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e)
        out_pooled[(long)b * d + (long)c * VEC + e] = h[e];
}

}  // namespace

// workgroups a unit's features are spread over: one 16-byte chunk per thread
static unsigned pool_feature_split(int d, bool bf16)
{
    const int nchunk = d / (bf16 ? 8 : 4);
    const int n = (nchunk + 255) / 256;
    return (unsigned)(n < 1 ? 1 : (n > 64 ? 64 : n));
}

hipError_t scan_lengths(const int32_t *lengths, int32_t B, int32_t *offsets, hipStream_t st)
{
    hipLaunchKernelGGL(scan_kernel<false>, dim3(1), dim3(256), 0, st, lengths, B, offsets);
    return hipGetLastError();
}

hipError_t segment_ids(const int32_t *offsets, int32_t B, int64_t T, int32_t *seg, hipStream_t st)
{
    if (T <= 0)
        return hipSuccess;
    hipLaunchKernelGGL(seg_ids_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, offsets, B,
                       (long)T, seg);
    return hipGetLastError();
}

hipError_t pool_entropy_weighted(const PoolArgs &a, hipStream_t st)
{
    if (a.B <= 0)
        return hipSuccess;
    const bool bf16 = a.dtype == DT_BF16;
    if (a.offsets == nullptr) {  // one new token per sequence, folded in place
        if (bf16)
            hipLaunchKernelGGL(plp_fold1_kernel<true>, dim3(a.B), dim3(256), 0, st, a.hidden, a.d, a.entropy,
                               a.k1_part, a.k1_nsplit, (long)a.T, a.slot, a.inv_alpha, a.out_pooled, a.out_lse);
        else
            hipLaunchKernelGGL(plp_fold1_kernel<false>, dim3(a.B), dim3(256), 0, st, a.hidden, a.d, a.entropy,
                               a.k1_part, a.k1_nsplit, (long)a.T, a.slot, a.inv_alpha, a.out_pooled, a.out_lse);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(scan_kernel<true>, dim3(1), dim3(256), 0, st, a.offsets, a.B, a.unit_start);
    hipLaunchKernelGGL(pool_lse_kernel, dim3(a.B), dim3(256), 0, st, a.entropy, a.offsets, (long)a.T, a.slot,
                       a.inv_alpha, a.state_lse, a.lse_new, a.state_scale);
    const long units = pool_units_bound(a.T, a.B);
    if (units > 0x7fffffffL)
        return hipErrorInvalidValue;
    const unsigned ysplit = pool_feature_split(a.d, bf16);
    if (units * ysplit > 0x7fffffffL)
        return hipErrorInvalidValue;
    if (bf16)
        hipLaunchKernelGGL((pool_partial_kernel<true, POOL_WEIGHTED>), dim3((unsigned)(units * ysplit)), dim3(256), 0, st, a.hidden,
                           a.d, a.entropy, a.offsets, a.B, (long)a.T, a.inv_alpha, a.lse_new, a.unit_start, (int)ysplit, a.partial);
    else
        hipLaunchKernelGGL((pool_partial_kernel<false, POOL_WEIGHTED>), dim3((unsigned)(units * ysplit)), dim3(256), 0, st, a.hidden,
                           a.d, a.entropy, a.offsets, a.B, (long)a.T, a.inv_alpha, a.lse_new, a.unit_start, (int)ysplit, a.partial);
    hipLaunchKernelGGL(pool_finalize_kernel, dim3(a.B, (a.d + 1023) / 1024), dim3(256), 0, st, a.partial,
                       a.unit_start, a.slot, a.d, (int)units, a.state_pooled, a.state_scale, a.lse_new, a.out_pooled,
                       a.out_lse);
    return hipGetLastError();
}

hipError_t pool_plain(const void *hidden, int dtype, int d, const int32_t *offsets, int32_t B, int64_t T,
                      int kind, int32_t *unit_start, float *partial, float *out_pooled, hipStream_t st)
{
    if (B <= 0)
        return hipSuccess;
    const bool bf16 = dtype == DT_BF16;
    if (kind == 2) {  // last token: one row per sequence
        const int vec = bf16 ? 8 : 4;
        const dim3 grid(B, (d / vec + 255) / 256);
        if (bf16)
            hipLaunchKernelGGL(pool_last_kernel<true>, grid, dim3(256), 0, st, hidden, d, offsets, (long)T,
                               out_pooled);
        else
            hipLaunchKernelGGL(pool_last_kernel<false>, grid, dim3(256), 0, st, hidden, d, offsets, (long)T,
                               out_pooled);
        return hipGetLastError();
    }
    // average and maximum stream every token once: same units of <= POOL_UNIT tokens as Eq. 4
    const long units = pool_units_bound(T, B);
    if (units > 0x7fffffffL)
        return hipErrorInvalidValue;
    const unsigned ysplit = pool_feature_split(d, bf16);
    if (units * ysplit > 0x7fffffffL)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(scan_kernel<true>, dim3(1), dim3(256), 0, st, offsets, B, unit_start);
    const dim3 fgrid(B, (d + 1023) / 1024);
#define EGTP_POOL_PLAIN(BF, MODE)                                                                          \
    do {                                                                                                   \
        hipLaunchKernelGGL((pool_partial_kernel<BF, MODE>), dim3((unsigned)(units * ysplit)), dim3(256), 0, st, hidden, \
                           d, nullptr, offsets, B, (long)T, 0.f, nullptr, unit_start, (int)ysplit, partial); \
        hipLaunchKernelGGL(pool_finalize_plain_kernel<MODE>, fgrid, dim3(256), 0, st, partial, unit_start, \
                           offsets, d, (int)units, out_pooled);                                            \
    } while (0)
    if (kind == 0) {
        if (bf16)
            EGTP_POOL_PLAIN(true, POOL_SUM);
        else
            EGTP_POOL_PLAIN(false, POOL_SUM);
    } else {
        if (bf16)
            EGTP_POOL_PLAIN(true, POOL_MAXIMUM);
        else
            EGTP_POOL_PLAIN(false, POOL_MAXIMUM);
    }
#undef EGTP_POOL_PLAIN
    return hipGetLastError();
}

}  // namespace egtp
