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
// Both operands are read from a PACKED copy: 256 rows x 32 K-elements per block of 16 KiB,
// stored exactly as the block sits in LDS (16-byte chunks XOR-swizzled by row so that the
// MFMA fragment reads are free of bank conflicts).  A K step of a tile is then one contiguous
// 16 KiB read, which is what HBM and the Infinity Cache want; reading 64-byte row pieces
// with a row stride of 2d bytes from the row-major matrices stalls the ring on DRAM page
// misses.  pack_rows_bf16 builds the packed copy (W_lm once, hidden states once per call;
// rows and K are zero-padded to whole blocks).
//
// Workgroup = 256 threads = 4 waves (2 along vocabulary x 2 along tokens), macro tile
// 256 vocabulary rows x 256 tokens, each wave 128 x 128 = 4x4 MFMA 32x32x16 tiles
// (256 accumulator registers).  Blocks go from global memory straight into an NSTAGE-deep
// LDS ring (16 bytes per lane, no staging registers).  One wave per SIMD means nothing
// hides a stall, so the instruction order inside a K step is pinned: every MFMA is followed
// by one load or one fragment read, which then issues in the shadow of the MFMA.  The one
// barrier per step sits between the two K sub-steps, after the reads of the current stage
// and before the fragments of the next step are fetched.
#include "kernels.h"

namespace egtp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

namespace {

constexpr int BM = 256;        // vocabulary rows per tile
constexpr int BN = 256;        // tokens per block
constexpr int BK = K1_PACK_K;  // K elements per step (32)
constexpr int ROW_BYTES = BK * 2;
constexpr int TILE_BYTES = 256 * ROW_BYTES;  // one operand block, 16 KiB
constexpr int STAGE_BYTES = 2 * TILE_BYTES;  // W block + hidden block
constexpr int NPASS = TILE_BYTES / 4096;     // 16-byte loads per lane and operand block (4)
constexpr int LOADS_PER_STEP = 2 * NPASS;
constexpr int TB_GROUP = 8;    // token blocks that sweep the same vocabulary range together
constexpr float NEG_BIG = -1.0e30f;
constexpr float LOG2E = 1.4426950408889634f;
static_assert(BK == 32 && TILE_BYTES == K1_PACK_BLOCK_BYTES, "packed block geometry");

struct Stats {
    float m, S, U;
};

// XOR key of a row's four 16-byte chunks inside a packed block (64-byte rows).  A fragment read
// takes the same logical chunk of consecutive rows; with this key any 16 consecutive rows fall
// on 16 different 16-byte bank groups of a 256-byte LDS line, and any 8 consecutive rows on 8
// different groups of a 128-byte line, so the reads are conflict-free either way.
__host__ __device__ __forceinline__ int swizzle_key(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

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
// statistics of that token.  MASK: only vocabulary rows < V count (the zero rows that pad
// the last tile are excluded).  row0 is the vocabulary row of element 0 for this lane.
template <bool MASK>
__device__ __forceinline__ void fold_tile(const f32x16 &a, Stats &st, int row0, int V)
{
    float z[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float v = a[i];
        if (MASK)
            v = (row0 + 8 * (i >> 2) + (i & 3)) < V ? v : NEG_BIG;
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

// scheduling-group masks of the AMDGPU backend
constexpr int SG_MFMA = 0x008, SG_VMEM_READ = 0x020, SG_DS_READ = 0x100;

template <int NSTAGE>
__global__ __launch_bounds__(256, 1) void k1_entropy_bf16_kernel(
    const unsigned char *__restrict__ Wp, const unsigned char *__restrict__ Hp, long T, int KT, int V,
    int ntb, int nsplit, int tps, int ntiles_v, float *__restrict__ part)
{
    static_assert(NSTAGE >= 3 && (NSTAGE - 2) * LOADS_PER_STEP < 64, "ring depth");
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave >> 1;  // vocabulary half of the macro tile
    const int wn = wave & 1;   // token half

    // ---- which (token block, vocabulary range) this workgroup owns -------------------
    // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous range of
    // logical units so that neighbours in time share W_lm blocks and token blocks in its L2.
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
    const int total = (vt_end - vt_begin) * KT;

    // ---- global -> LDS: a block is copied linearly, 1 KiB per wave-wide load ------------
    const unsigned lane_off = (unsigned)(wave * 1024 + lane * 16);
    const unsigned char *Hblk = Hp + (long)tb * KT * TILE_BYTES + lane_off;
    const unsigned char *Wl = Wp + lane_off;
    unsigned char *lds_wave = smem + wave * 1024;
    auto issue_loads = [&](int vt, int kt, int stage) {
        const unsigned char *Wt = Wl + ((long)vt * KT + kt) * TILE_BYTES;
        const unsigned char *Ht = Hblk + (long)kt * TILE_BYTES;
        unsigned char *dst = lds_wave + stage * STAGE_BYTES;
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            load16_to_lds(Wt + p * 4096, dst + p * 4096);
            load16_to_lds(Ht + p * 4096, dst + TILE_BYTES + p * 4096);
        }
    };

    // ---- fragment read geometry (row r, chunk c sits at r*64 + ((c ^ swizzle_key(r)) * 16)) ----
    const int l31 = lane & 31;
    const int khalf = lane >> 5;
    const unsigned fragA = (unsigned)(wm * 128 + l31) * ROW_BYTES;
    const unsigned fragB = (unsigned)TILE_BYTES + (unsigned)(wn * 128 + l31) * ROW_BYTES;
    const int swf = swizzle_key(l31);  // row = l31 + a multiple of 32
    const unsigned swz0 = (unsigned)(((0 + khalf) ^ swf) << 4);
    const unsigned swz1 = (unsigned)(((2 + khalf) ^ swf) << 4);

    Stats st[4];
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
        st[ni].m = NEG_BIG;
        st[ni].S = 0.f;
        st[ni].U = 0.f;
    }

    // The load stream runs NSTAGE-1 steps ahead of the MFMAs.  Past the end it keeps
    // re-reading the last step (same addresses, into a stage nobody reads any more), so
    // every step issues the same number of loads and one wait constant serves the sweep.
    int lvt = vt_begin, lkt = 0, lstep = 0;
    auto advance_ld = [&]() {  // branch-free: a step must stay one scheduling region
        const int adv = lstep + 1 < total ? 1 : 0;
        lstep += adv;
        const int nk = lkt + adv;
        const int wrap = nk == KT ? 1 : 0;
        lkt = wrap ? 0 : nk;
        lvt += wrap;
    };
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; ++s) {
        issue_loads(lvt, lkt, s);
        advance_ld();
    }
    wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();

    bf16x8 fa[2][4], fb[2][4];
#define EGTP_READ_FRAGS(set_, stage_base_, swz_)                                                  \
    {                                                                                             \
        _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                          \
            fa[set_][mi] = *(const bf16x8 *)((stage_base_) + fragA + mi * 32 * ROW_BYTES + swz_); \
        _Pragma("unroll") for (int ni = 0; ni < 4; ++ni)                                          \
            fb[set_][ni] = *(const bf16x8 *)((stage_base_) + fragB + ni * 32 * ROW_BYTES + swz_); \
    }
#define EGTP_MFMA_PHASE(set_)                                                                     \
    {                                                                                             \
        _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                          \
            _Pragma("unroll") for (int ni = 0; ni < 4; ++ni)                                      \
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set_][mi], fb[set_][ni], \
                                                                      acc[mi][ni], 0, 0, 0);      \
    }
    EGTP_READ_FRAGS(0, smem, swz0);

    int ldstage = NSTAGE - 1;  // stage the next loads go to
    int cstage = 0;            // stage being consumed
    for (int vt = vt_begin; vt < vt_end; ++vt) {
        f32x16 acc[4][4];
#pragma unroll
        for (int mi = 0; mi < 4; ++mi)
#pragma unroll
            for (int ni = 0; ni < 4; ++ni)
#pragma unroll
                for (int i = 0; i < 16; ++i)
                    acc[mi][ni][i] = 0.f;

        for (int kt = 0; kt < KT; ++kt) {
            const unsigned char *sA = smem + cstage * STAGE_BYTES;
            const int nstage = cstage + 1 == NSTAGE ? 0 : cstage + 1;
            const unsigned char *sN = smem + nstage * STAGE_BYTES;
            // ---- first half: loads for the step NSTAGE-1 ahead (into the stage consumed in
            //      the previous step), fragments of sub-step 1, MFMAs of sub-step 0
            issue_loads(lvt, lkt, ldstage);
            advance_ld();
            ldstage = ldstage + 1 == NSTAGE ? 0 : ldstage + 1;
            EGTP_READ_FRAGS(1, sA, swz1);
            EGTP_MFMA_PHASE(0);
#pragma unroll
            for (int j = 0; j < LOADS_PER_STEP; ++j) {
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
                __builtin_amdgcn_sched_group_barrier(SG_VMEM_READ, 1, 0);
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
                __builtin_amdgcn_sched_group_barrier(SG_DS_READ, 1, 0);
            }
            // ---- the next step's blocks have landed (own loads; the newest NSTAGE-2 steps may
            //      still be in flight), then everyone's.  Every read of the current stage has
            //      been consumed by now.  A bare barrier: a fence would drain the whole ring.
            wait_vmcnt<(NSTAGE - 2) * LOADS_PER_STEP>();
            __builtin_amdgcn_s_barrier();
            // ---- second half: fragments of the next step's sub-step 0, MFMAs of sub-step 1
            EGTP_READ_FRAGS(0, sN, swz0);
            EGTP_MFMA_PHASE(1);
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);
                __builtin_amdgcn_sched_group_barrier(SG_DS_READ, 1, 0);
            }
            cstage = nstage;
        }

        // a full tile of logits is in registers: fold it into the statistics and forget it
        const int row_base = vt * BM + wm * 128 + 4 * khalf;
        if (vt * BM + BM > V) {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    fold_tile<true>(acc[mi][ni], st[ni], row_base + mi * 32, V);
        } else {
#pragma unroll
            for (int mi = 0; mi < 4; ++mi)
#pragma unroll
                for (int ni = 0; ni < 4; ++ni)
                    fold_tile<false>(acc[mi][ni], st[ni], row_base + mi * 32, V);
        }
    }
#undef EGTP_READ_FRAGS
#undef EGTP_MFMA_PHASE

    // drain the ring (the tail re-reads) before its memory is reused
    wait_vmcnt<0>();
    __syncthreads();

    // ---- combine the lanes and waves that hold the same token ----------------------------
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
        Stats o;
        o.m = __shfl_xor(st[ni].m, 32);
        o.S = __shfl_xor(st[ni].S, 32);
        o.U = __shfl_xor(st[ni].U, 32);
        st[ni] = merge(st[ni], o);
    }
    float *red = (float *)smem;  // [wn][ni][32][3]
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

// The same merge for many ranges per token (small batches split the vocabulary finely): one
// wave per token, lane l takes ranges l, l+64, ... in order, then a fixed xor tree joins the
// lanes -- still a fixed order, so bit-reproducible.
__global__ __launch_bounds__(256) void k1_merge_wide_kernel(const float *__restrict__ part, int nsplit,
                                                            long T, float *__restrict__ entropy)
{
    const long t = (long)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int lane = threadIdx.x & 63;
    if (t >= T)
        return;
    const long plane = (long)nsplit * T;
    Stats a;
    a.m = NEG_BIG;
    a.S = 0.f;
    a.U = 0.f;
    for (int s = lane; s < nsplit; s += 64) {
        Stats b;
        const long idx = (long)s * T + t;
        b.m = part[idx];
        b.S = part[plane + idx];
        b.U = part[2 * plane + idx];
        a = merge(a, b);
    }
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        Stats b;
        b.m = __shfl_xor(a.m, o);
        b.S = __shfl_xor(a.S, o);
        b.U = __shfl_xor(a.U, o);
        a = merge(a, b);
    }
    if (lane == 0)
        entropy[t] = logf(a.S) - a.U * 0.6931471805599453f / a.S;
}

// Packs rows of a row-major bf16 matrix src[R x d] into blocks of 256 rows x 32 K-elements in
// LDS-image order; rows >= R and K >= d are zero.  One workgroup packs 8 consecutive K steps
// of one row tile: a wave reads 512 contiguous bytes of each of two rows at a time.
__global__ __launch_bounds__(256) void pack_rows_bf16_kernel(const unsigned char *__restrict__ src, long R,
                                                             int d, int KT, unsigned char *__restrict__ dst)
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
    for (int r = rsub; r < 256; r += 8) {
        const long row = tile * 256 + r;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (row < R && k_elem < d)
            v = *(const uint4 *)(src + (row * d + k_elem) * 2);
        *(uint4 *)(blk + r * ROW_BYTES + ((chunk ^ swizzle_key(r)) << 4)) = v;
    }
}

}  // namespace

size_t k1_packed_bytes(int64_t rows, int d)
{
    const int64_t tiles = (rows + 255) / 256;
    const int64_t kt = (d + BK - 1) / BK;
    return (size_t)(tiles * kt) * TILE_BYTES;
}

hipError_t k1_pack_rows_bf16(const void *src, int64_t rows, int d, void *dst, hipStream_t st)
{
    if (rows <= 0)
        return hipSuccess;
    const long tiles = (rows + 255) / 256;
    const int kt = (d + BK - 1) / BK;
    if (tiles > 0x7fffffffL)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(pack_rows_bf16_kernel, dim3((unsigned)tiles, (kt + 7) / 8), dim3(256), 0, st,
                       (const unsigned char *)src, (long)rows, d, kt, (unsigned char *)dst);
    return hipGetLastError();
}

hipError_t k1_entropy_bf16(const void *hidden_packed, const void *w_packed, int64_t T, int d, int V,
                           const K1Plan &p, float *part, hipStream_t st)
{
    constexpr int NSTAGE = 4;
    constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)k1_entropy_bf16_kernel<NSTAGE>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
        if (e != hipSuccess)
            return e;
        attr_set = true;
    }
    if (p.tb_tokens != BN || p.tile_v != BM || T <= 0)
        return hipErrorInvalidValue;
    const long units = (long)p.ntb * p.nsplit;
    if (units <= 0 || units > 0x7fffffffL)
        return hipErrorInvalidValue;
    const int kt = (d + BK - 1) / BK;
    hipLaunchKernelGGL((k1_entropy_bf16_kernel<NSTAGE>), dim3((unsigned)units), dim3(256), LDS_BYTES, st,
                       (const unsigned char *)w_packed, (const unsigned char *)hidden_packed, (long)T, kt, V,
                       p.ntb, p.nsplit, p.tiles_per_split, p.ntiles_v, part);
    return hipGetLastError();
}

hipError_t k1_merge(const float *part, int nsplit, int64_t T, float *entropy, hipStream_t st)
{
    if (nsplit >= 32) {
        const long wblocks = (T + 3) / 4;
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
