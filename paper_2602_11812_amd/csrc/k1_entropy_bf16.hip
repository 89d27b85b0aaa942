// Fused LM-head contraction + streaming entropy for bf16 inputs on gfx950 (Eq. 2).
//
// logits^T = W_lm . hidden^T is computed tile by tile on the bf16 matrix cores with the
// vocabulary as the MFMA row dimension and the tokens as its column dimension.  With the
// 32x32 accumulator layout every lane then holds logits of ONE token (its column) for
// 16 vocabulary rows per MFMA tile, so the softmax statistics of a token
//     m = max z,  S = sum e^{z-m},  U = sum e^{z-m} (z-m) log2(e)
// are carried in registers, lane-private, across the whole vocabulary sweep, and lanes are
// only combined once at the end.  Logits never leave the register file:
// H = ln S - U ln2 / S  is finished by the merge kernel from one triple per
// (token, vocabulary range).
//
// Workgroup = 256 threads = 4 waves (2 along vocabulary x 2 along tokens), macro tile
// 256 vocabulary rows x 256 tokens, each wave 128 x 128 = 4x4 MFMA 32x32x16 tiles
// (256 accumulator registers).  Operand tiles go from global memory straight into LDS
// (16 bytes per lane, no staging registers) through an NSTAGE-deep ring of K steps;
// 16-byte chunks are XOR-swizzled by row so that the MFMA fragment reads are conflict-free.
#include "kernels.h"

namespace egtp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int BM = 256;      // vocabulary rows per tile
constexpr int BN = 256;      // tokens per block
constexpr int TB_GROUP = 8;  // token blocks that sweep the same vocabulary range together
constexpr float NEG_BIG = -1.0e30f;
constexpr float LOG2E = 1.4426950408889634f;

struct Stats {
    float m, S, U;
};

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// (m1,S1,U1) (+) (m2,S2,U2): statistics of the union of two disjoint sets of logits
__device__ __forceinline__ Stats merge(Stats a, Stats b)
{
    float M = fmaxf(a.m, b.m);
    float da = (a.m - M) * LOG2E, db = (b.m - M) * LOG2E;
    float sa = fast_exp2(da), sb = fast_exp2(db);
    Stats r;
    r.m = M;
    r.S = a.S * sa + b.S * sb;
    r.U = (a.U + da * a.S) * sa + (b.U + db * b.S) * sb;
    return r;
}

// Fold the 16 logits a lane holds for one token column in one MFMA tile into the running
// statistics of that token.  MASK: only vocabulary rows >= row_lo count (the last tile of a
// ragged vocabulary is loaded shifted back so that it ends at V; its leading rows belong to
// the tile before).  row0 is the vocabulary row of element 0 for this lane.
template <bool MASK>
__device__ __forceinline__ void fold_tile(const f32x16 &a, Stats &st, int row0, int row_lo)
{
    float z[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float v = a[i];
        if (MASK)
            v = (row0 + 8 * (i >> 2) + (i & 3)) >= row_lo ? v : NEG_BIG;
        z[i] = v;
    }
    float mx = z[0];
#pragma unroll
    for (int i = 1; i < 16; ++i)
        mx = fmaxf(mx, z[i]);
    if (MASK && !(mx > NEG_BIG))
        return;  // every row of this lane is masked: nothing to add (and no reference maximum yet)
    if (mx > st.m) {  // new running maximum: rescale what has been summed so far
        float dl = (st.m - mx) * LOG2E;
        float sc = fast_exp2(dl);
        st.U = (st.U + dl * st.S) * sc;
        st.S = st.S * sc;
        st.m = mx;
    }
    const float mc = -st.m * LOG2E;
    float S0 = 0.f, S1 = 0.f, U0 = 0.f, U1 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; i += 2) {
        float t0 = fmaf(z[i], LOG2E, mc);
        float t1 = fmaf(z[i + 1], LOG2E, mc);
        float e0 = fast_exp2(t0);
        float e1 = fast_exp2(t1);
        S0 += e0;
        S1 += e1;
        U0 = fmaf(e0, t0, U0);
        U1 = fmaf(e1, t1, U1);
    }
    st.S += S0 + S1;
    st.U += U0 + U1;
}

// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits
// [3:0] and [15:14], export and LDS/scalar counters left at their maxima)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// 16 bytes per lane from global memory straight into LDS: lane i of the wave lands at
// lds_wave_base + 16 * i.
__device__ __forceinline__ void load16_to_lds(const unsigned char *g, unsigned char *lds_wave_base)
{
    __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)g,
                                     (__attribute__((address_space(3))) void *)lds_wave_base, 16, 0, 0);
}

template <int BK, int NSTAGE>
__global__ __launch_bounds__(256, 1) void k1_entropy_bf16_kernel(
    const unsigned char *__restrict__ Wb, const unsigned char *__restrict__ Hb, long T, int d, int V,
    int ntb, int nsplit, int tps, int ntiles_v, float *__restrict__ part)
{
    constexpr int ROW_BYTES = BK * 2;             // bytes of one tile row in LDS
    constexpr int CPR = ROW_BYTES / 16;           // 16-byte chunks per row (8 or 4)
    constexpr int TILE_BYTES = 256 * ROW_BYTES;   // one operand tile
    constexpr int STAGE_BYTES = 2 * TILE_BYTES;   // A + B
    constexpr int ROWS_PER_WAVE_LOAD = 64 / CPR;  // rows covered by one wave-wide 1 KiB load
    constexpr int NPASS = 256 / (4 * ROWS_PER_WAVE_LOAD);  // loads per lane, operand and K step
    constexpr int KK = BK / 16;                   // MFMA K sub-steps per K step
    constexpr int LOADS_PER_STEP = 2 * NPASS;
    static_assert(BK == 64 || BK == 32, "K step");
    static_assert((NSTAGE - 2) * LOADS_PER_STEP < 64, "vmcnt range");

    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1;  // vocabulary half of the macro tile
    const int wn = wave & 1;   // token half

    // ---- which (token block, vocabulary range) this workgroup owns -------------------
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
    // logical units so that neighbours in time share W_lm tiles and token blocks in its L2.
    int tb, sp;
    {
        const int units = gridDim.x;
        const int id = blockIdx.x;
        const int q = units >> 3, r = units & 7;
        const int x = id & 7, j = id >> 3;
        const int logical = x * q + (x < r ? x : r) + j;
        const int per_group = TB_GROUP * nsplit;
        const int g = logical / per_group;
        const int rem = logical - g * per_group;
        const int gsize = min(TB_GROUP, ntb - g * TB_GROUP);
        sp = rem / gsize;
        tb = g * TB_GROUP + (rem - sp * gsize);
    }
    const int vt_begin = sp * tps;
    const int vt_end = min(ntiles_v, vt_begin + tps);
    const long tok0 = (long)tb * BN;
    const long row_bytes = (long)d * 2;
    const int KT = d / BK;  // d is a multiple of BK (checked by the launcher)

    // ---- global -> LDS geometry ----------------------------------------------------------
    // One wave-wide load fills 1 KiB of LDS = ROWS_PER_WAVE_LOAD rows; pass p of wave w fills
    // rows (p*4 + w) * ROWS_PER_WAVE_LOAD ...  Lane l sits at row lr = l / CPR, chunk slot
    // l % CPR of that block and therefore fetches the logical chunk (slot ^ swizzle(row)).
    const int lr = lane / CPR;
    const int slot = lane % CPR;
    const int row_in_tile0 = wave * ROWS_PER_WAVE_LOAD + lr;  // + p * 4 * ROWS_PER_WAVE_LOAD
    const int sw0 = CPR == 8 ? (row_in_tile0 & 7) : ((row_in_tile0 >> 1) & 3);
    const unsigned chunk_bytes = (unsigned)((slot ^ sw0) * 16);
    // (p * 4 * ROWS_PER_WAVE_LOAD is a multiple of 16, so the swizzle term does not depend on p)
    const unsigned offA0 = (unsigned)(row_in_tile0 * row_bytes) + chunk_bytes;
    const long passA = (long)(4 * ROWS_PER_WAVE_LOAD) * row_bytes;
    const unsigned char *Hblk = Hb + tok0 * row_bytes;
    unsigned offB[NPASS];
    {
        const long last = T - 1 - tok0;  // >= 0: the block holds at least one token
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            long rr = row_in_tile0 + p * 4 * ROWS_PER_WAVE_LOAD;
            rr = rr < last ? rr : last;  // rows past the end re-read the last token (discarded)
            offB[p] = (unsigned)(rr * row_bytes) + chunk_bytes;
        }
    }
    unsigned char *lds_wave = smem + wave * 1024;  // + stage * STAGE_BYTES + p * 4096 (+ TILE_BYTES for B)

    // tile vt starts at vocabulary row min(vt * BM, V - BM): the last tile of a ragged
    // vocabulary is shifted back (V >= BM is checked by the launcher)
    auto issue_loads = [&](int vt, int kt, int stage) {
        const int v0 = min(vt * BM, V - BM);
        const unsigned char *Wt = Wb + (long)v0 * row_bytes + (long)kt * ROW_BYTES;
        const unsigned char *Ht = Hblk + (long)kt * ROW_BYTES;
        unsigned char *dst = lds_wave + stage * STAGE_BYTES;
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            load16_to_lds(Wt + p * passA + offA0, dst + p * 4096);
            load16_to_lds(Ht + offB[p], dst + TILE_BYTES + p * 4096);
        }
    };

    // ---- fragment read geometry --------------------------------------------------------
    const int l31 = lane & 31;
    const int khalf = lane >> 5;
    const unsigned fragA = (unsigned)(wm * 128 + l31) * ROW_BYTES;
    const unsigned fragB = (unsigned)TILE_BYTES + (unsigned)(wn * 128 + l31) * ROW_BYTES;
    const int swf = CPR == 8 ? (l31 & 7) : ((l31 >> 1) & 3);
    unsigned swz[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk)
        swz[kk] = (unsigned)(((kk * 2 + khalf) ^ swf) << 4);

    Stats st[4];
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
        st[ni].m = NEG_BIG;
        st[ni].S = 0.f;
        st[ni].U = 0.f;
    }

    const int total = (vt_end - vt_begin) * KT;

    // ---- prologue: fill NSTAGE-1 stages -------------------------------------------------
    int lvt = vt_begin, lkt = 0, lstep = 0;  // the load stream's position
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) {
        if (lstep < total) {
            issue_loads(lvt, lkt, s);
            ++lstep;
            if (++lkt == KT) {
                lkt = 0;
                ++lvt;
            }
        }
    }
    if (total <= NSTAGE - 1)
        wait_vmcnt<0>();
    else
        wait_vmcnt<(NSTAGE - 2) * LOADS_PER_STEP>();
    __builtin_amdgcn_s_barrier();

    int it = 0;
    for (int vt = vt_begin; vt < vt_end; ++vt) {
        f32x16 acc[4][4];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    acc[mi][ni][i] = 0.f;

        for (int kt = 0; kt < KT; ++kt, ++it) {
            // refill the stage that was consumed in the previous iteration
            if (lstep < total) {
                issue_loads(lvt, lkt, lstep % NSTAGE);
                ++lstep;
                if (++lkt == KT) {
                    lkt = 0;
                    ++lvt;
                }
            }
            const unsigned char *sA = smem + (it % NSTAGE) * STAGE_BYTES;
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                bf16x8 af[4], bfr[4];
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
                    af[mi] = *(const bf16x8 *)(sA + fragA + mi * 32 * ROW_BYTES + swz[kk]);
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    bfr[ni] = *(const bf16x8 *)(sA + fragB + ni * 32 * ROW_BYTES + swz[kk]);
#pragma unroll
                for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                    for (int ni = 0; ni < 4; ++ni)
                        acc[mi][ni] =
                            __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
            }
            // the next step's tile must have landed (own loads), then everyone's
            if (lstep - (it + 1) >= NSTAGE - 1)
                wait_vmcnt<(NSTAGE - 2) * LOADS_PER_STEP>();
            else
                wait_vmcnt<0>();
            // A bare barrier: every LDS read of this step has already been consumed by an
            // MFMA, and the direct-to-LDS loads are ordered by the explicit counter waits
            // above, so no memory fence (which would drain the whole load ring) is needed.
            __builtin_amdgcn_s_barrier();
        }

        // a full tile of logits is in registers: fold it into the statistics and forget it
        const int v0 = min(vt * BM, V - BM);
        const int row_base = v0 + wm * 128 + 4 * khalf;
        const int row_lo = vt * BM;
        if (v0 < row_lo) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    fold_tile<true>(acc[mi][ni], st[ni], row_base + mi * 32, row_lo);
        } else {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    fold_tile<false>(acc[mi][ni], st[ni], row_base + mi * 32, row_lo);
        }
    }

    // ---- combine the lanes and waves that hold the same token ----------------------------
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
        Stats o;
        o.m = __shfl_xor(st[ni].m, 32);
        o.S = __shfl_xor(st[ni].S, 32);
        o.U = __shfl_xor(st[ni].U, 32);
        st[ni] = merge(st[ni], o);
    }
    float *red = (float *)smem;  // [wn][ni][32][3]; the main loop ended on a barrier
    if (wm == 1 && lane < 32) {
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            float *r = red + ((wn * 4 + ni) * 32 + lane) * 3;
            r[0] = st[ni].m;
            r[1] = st[ni].S;
            r[2] = st[ni].U;
        }
    }
    __syncthreads();
    if (wm == 0 && lane < 32) {
        const long plane = (long)nsplit * T;
#pragma unroll
        for (int ni = 0; ni < 4; ++ni) {
            const float *r = red + ((wn * 4 + ni) * 32 + lane) * 3;
            Stats o;
            o.m = r[0];
            o.S = r[1];
            o.U = r[2];
            Stats f = merge(st[ni], o);
            const long tok = tok0 + wn * 128 + ni * 32 + lane;
            if (tok < T) {
                const long idx = (long)sp * T + tok;
                part[idx] = f.m;
                part[plane + idx] = f.S;
                part[2 * plane + idx] = f.U;
            }
        }
    }
}

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

template <int BK, int NSTAGE>
hipError_t launch(const void *hidden, const void *w_lm, int64_t T, int d, int V, const K1Plan &p, float *part,
                  hipStream_t st)
{
    constexpr int LDS_BYTES = NSTAGE * 2 * 256 * BK * 2;
    static_assert(LDS_BYTES <= 160 * 1024, "LDS budget");
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k1_entropy_bf16_kernel<BK, NSTAGE>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess)
            return e;
        attr_set = true;
    }
    const long units = (long)p.ntb * p.nsplit;
    hipLaunchKernelGGL((k1_entropy_bf16_kernel<BK, NSTAGE>), dim3((unsigned)units), dim3(256), LDS_BYTES, st,
                       (const unsigned char *)w_lm, (const unsigned char *)hidden, (long)T, d, V, p.ntb,
                       p.nsplit, p.tiles_per_split, p.ntiles_v, part);
    return hipGetLastError();
}

}  // namespace

bool k1_bf16_mfma_supported(int d, int V) { return d % 64 == 0 && V >= BM; }

hipError_t k1_entropy_bf16(const void *hidden, const void *w_lm, int64_t T, int d, int V,
                           const K1Plan &p, float *part, hipStream_t st)
{
    if (p.tb_tokens != BN || p.tile_v != BM || !k1_bf16_mfma_supported(d, V) || T <= 0)
        return hipErrorInvalidValue;
    const long units = (long)p.ntb * p.nsplit;
    if (units <= 0 || units > 0x7fffffffL)
        return hipErrorInvalidValue;
    switch (p.variant) {
    case 1: return launch<32, 4>(hidden, w_lm, T, d, V, p, part, st);
    case 2: return launch<32, 3>(hidden, w_lm, T, d, V, p, part, st);
    default: return launch<64, 2>(hidden, w_lm, T, d, V, p, part, st);
    }
}

hipError_t k1_merge(const float *part, int nsplit, int64_t T, float *entropy, hipStream_t st)
{
    const long blocks = (T + 255) / 256;
    if (blocks <= 0 || blocks > 0x7fffffffL)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k1_merge_kernel, dim3((unsigned)blocks), dim3(256), 0, st, part, nsplit,
                       (long)T, entropy);
    return hipGetLastError();
}

}  // namespace egtp
