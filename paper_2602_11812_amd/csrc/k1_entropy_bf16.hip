// Fused LM-head contraction + streaming entropy on the bf16 matrix cores of gfx950 (Eq. 2).  bf16 inputs
// are contracted as they are; fp32 inputs arrive split into bf16 pieces laid side by side along K (see the
// packing kernels), so the same kernel gives fp32-grade logits from a contraction six times as long.
//
// logits^T = W_lm . hidden^T is computed tile by tile on the bf16 matrix cores with the
// vocabulary as the MFMA row dimension and the tokens as its column dimension.  In the
// 16x16 accumulator layout a lane holds rows 4*(l/16)+i of column l%16, i.e. logits of ONE
// token (its column), so the softmax statistics of a token
//     m = max z (kept in log2 units),  S = sum e^{z-m},  U = sum e^{z-m} (z-m) log2(e)
// are carried in registers, lane-private, across the whole vocabulary sweep, and the four
// lanes and two waves that share a token are only combined once at the end.  Logits never
// leave the register file:  H = ln S - U ln2 / S  is finished by the merge kernel from one
// triple per (token, vocabulary range).
//
// Both operands are read from a PACKED copy: 256 rows x 32 K-elements per block of 16 KiB,
// stored exactly as the block sits in LDS (16-byte chunks XOR-swizzled by row so that the
// MFMA fragment reads are free of bank conflicts).  A K step of a tile is then one contiguous
// 16 KiB read, which is what HBM and the Infinity Cache want; reading 64-byte row pieces
// with a row stride of 2d bytes from the row-major matrices stalls the ring on DRAM page
// misses.  The packing kernels build the packed copy (W_lm once, hidden states once per call;
// rows are zero-padded to whole blocks, K to an even number of blocks).
//
// Workgroup = 256 threads = 4 waves (2 along vocabulary x 2 along tokens), macro tile
// 256 vocabulary rows x 256 tokens, each wave 128 x 128 = 8x8 MFMA 16x16x32 tiles
// (256 accumulator registers); one 16-byte fragment read covers a whole K step: lane l
// holds row l%16, chunk l/16 of the 64-byte row.  Blocks go from global memory straight
// into an NSTAGE-deep LDS ring (buffer loads to LDS, 16 bytes per lane, no staging registers).  The kernel runs
// at the package power limit, so what counts is energy per FLOP: the 16x16x32 shape with the
// first operand held for 8 consecutive MFMAs (row-major tile order) draws markedly less
// power than 32x32x16 or than any order that changes both operands every MFMA.  One wave
// per SIMD means nothing hides a stall, so the instruction order inside a K step is pinned:
// loads and fragment reads are spread between the MFMAs, which cover them.  The one barrier
// per step sits between the step's two halves, after the last read of the current stage.
//
// Pacing.  The 32 workgroups that run on one XCD at a time cover 8 token blocks x 4 vocabulary
// ranges and read every block they share from the XCD's L2 -- as long as they walk through K
// together.  Left alone they drift apart and the L2 (4 MiB, about 20 K steps of their blocks)
// misses; the extra traffic over the fabric costs power, and power is the limit.  So every
// PACE_TILES vocabulary tiles each workgroup counts itself in on a counter of its cohort and
// the early ones wait for the rest.  The wait is a hint, not a dependency: it is bounded, a
// workgroup whose wait runs out stops pacing for good, and no result depends on it.
#include "k1_common.h"

namespace egtp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

namespace {

constexpr int BM = 256;        // vocabulary rows per tile
constexpr int BN = 256;        // tokens per block
constexpr int STAGE_BYTES = 2 * TILE_BYTES;  // W block + hidden block
constexpr int NPASS = TILE_BYTES / 4096;     // 16-byte loads per lane and operand block (4)
constexpr int LOADS_PER_STEP = 2 * NPASS;
constexpr int TB_GROUP = 8;    // token blocks that sweep the same vocabulary range together
constexpr int XCDS = 8;            // workgroup i is placed on XCD i % 8
constexpr int COHORT = 32;         // workgroups one XCD runs at a time (its compute units)
constexpr int PACE_TILES = K1_PACE_TILES;  // vocabulary tiles between two pacing points
constexpr int PACE_SPINS = 24;     // bound of one wait: polls of the counter ...
constexpr int PACE_SLEEP = 4;      // ... each followed by a sleep of 64 * PACE_SLEEP cycles
// s_waitcnt with only the vector-memory counter constrained (gfx9 encoding: vmcnt in bits
// [3:0] and [15:14], export and LDS/scalar counters left at their maxima)
template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// 16 bytes per lane from memory straight into LDS: lane i of the wave lands at lds_wave_base + 16 * i.
// A buffer load (descriptor + per-lane byte offset + scalar byte offset): the address of a K step is then one
// scalar add, with no 64-bit vector arithmetic in the main loop, and the hardware clamps every access to the
// descriptor's range.  Measured against the flat-address form of the same load: 0.5 % faster.
__device__ __forceinline__ void load16_to_lds(__amdgpu_buffer_rsrc_t rsrc, int lane_byte_offset, int scalar_byte_offset,
                                              unsigned char *lds_wave_base)
{
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (__attribute__((address_space(3))) void *)lds_wave_base, 16,
                                             lane_byte_offset, scalar_byte_offset, 0, 0);
}
// raw buffer descriptor over `bytes` bytes at p (gfx9 family: 32-bit data format word, no swizzle)
__device__ __forceinline__ __amdgpu_buffer_rsrc_t raw_buffer(const unsigned char *p, int bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc((void *)p, 0, bytes, 0x00020000);
}

// scheduling-group masks of the AMDGPU backend
constexpr int SG_MFMA = 0x008, SG_VMEM_READ = 0x020, SG_DS_READ = 0x100;

// Fold 16 logits of one token: zin[4*q+i] is vocabulary row row0 + 16*q + i.
template <bool MASK>
__device__ __forceinline__ void fold16(const float (&zin)[16], Stats &st, int row0, int V)
{
    float z[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        float v = zin[i];
        if (MASK)
            v = (row0 + 16 * (i >> 2) + (i & 3)) < V ? v : NEG_BIG;
        z[i] = v;
    }
    float mx = z[0];
#pragma unroll
    for (int i = 1; i < 16; ++i)
        mx = fmaxf(mx, z[i]);
    if (MASK && !(mx > NEG_BIG))
        return;  // every row of this lane is masked: nothing to add (and no reference maximum yet)
    // The reference lives in log2 units, r = fl(max z * log2 e): every exponent is then ONE fused
    // multiply-add z * log2 e - r (exact product, one rounding of a small result) and re-referencing is an
    // exact difference of two r, so the precision does not degrade with the magnitude of the logits.
    const float r = mx * LOG2E;
    if (r > st.m) {  // new running reference: rescale what has been summed so far
        float dl = st.m - r;
        float sc = fast_exp2(dl);
        st.U = (st.U + dl * st.S) * sc;
        st.S = st.S * sc;
        st.m = r;
    }
    const float mc = -st.m;
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

__global__ void k1_pace_zero_kernel(int *__restrict__ pace, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n)
        pace[i] = 0;
}

template <int NSTAGE>
__global__ __launch_bounds__(256, 1) void k1_entropy_bf16_kernel(
    const unsigned char *__restrict__ Wp, const unsigned char *__restrict__ Hp, long T, int KT, int V,
    int ntb, int nsplit, int tps, int ntiles_v, float *__restrict__ part, int *__restrict__ pace)
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
    int *pace_cnt = nullptr;  // this workgroup's cohort counter (thread 0 only), or NULL: no pacing
    int pace_members = 0;
    {
        const int units = gridDim.x;
        const int id = blockIdx.x;
        const int q = units >> 3, r = units & 7;
        const int x = id & 7, j = id >> 3;
        // cohort = 32 consecutive workgroups of one XCD (the ones it starts together)
        if (pace != nullptr && tid == 0) {
            const int cohort = j / COHORT;
            pace_cnt = pace + x * k1_pace_cohorts(units) + cohort;
            pace_members = min(COHORT, q + (x < r ? 1 : 0) - cohort * COHORT);
        }
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
    const int lane_off = wave * 1024 + lane * 16;
    const int tile_bytes = KT * TILE_BYTES;  // one row tile of a packed operand over all of K (the launcher checks the range)
    const __amdgpu_buffer_rsrc_t rH = raw_buffer(Hp + (long)tb * tile_bytes, tile_bytes);  // this workgroup's token block
    unsigned char *lds_wave = smem + wave * 1024;
    auto issue_loads = [&](int vt, int kt, int stage) {
        // the descriptor of W_lm moves with the vocabulary tile, so that byte offsets stay inside one tile
        const __amdgpu_buffer_rsrc_t rW = raw_buffer(Wp + (long)vt * tile_bytes, tile_bytes);
        const int koff = kt * TILE_BYTES;
        unsigned char *dst = lds_wave + stage * STAGE_BYTES;
#pragma unroll
        for (int p = 0; p < NPASS; ++p) {
            load16_to_lds(rW, lane_off, koff + p * 4096, dst + p * 4096);
            load16_to_lds(rH, lane_off, koff + p * 4096, dst + TILE_BYTES + p * 4096);
        }
    };

    // ---- fragment read geometry: row r, chunk c sits at r*64 + ((c ^ swizzle_key(r)) * 16); the key
    //      of row 16*t + l15 is the key of l15
    const int l15 = lane & 15;
    const int kq = lane >> 4;
    const unsigned swz = (unsigned)((kq ^ swizzle_key(l15)) << 4);
    const unsigned fragA = (unsigned)(wm * 128 + l15) * ROW_BYTES + swz;
    const unsigned fragB = (unsigned)TILE_BYTES + (unsigned)(wn * 128 + l15) * ROW_BYTES + swz;
    constexpr int FRAG_STRIDE = 16 * ROW_BYTES;  // 16 rows further

    Stats st[8];
#pragma unroll
    for (int ni = 0; ni < 8; ++ni) {
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

    // Fragments of the current step: rows 0..63 (fa0) and 64..127 (fa1) of the wave tile, re-read in
    // place once their half is done, and two sets of 8 column fragments that swap roles every step.
    bf16x8 fa0[4], fa1[4], fbA[8], fbB[8];
#pragma unroll
    for (int i = 0; i < 4; ++i)
        fa0[i] = *(const bf16x8 *)(smem + fragA + i * FRAG_STRIDE);
#pragma unroll
    for (int i = 0; i < 8; ++i)
        fbA[i] = *(const bf16x8 *)(smem + fragB + i * FRAG_STRIDE);

    int ldstage = NSTAGE - 1;  // stage the next loads go to
    int cstage = 0;            // stage being consumed
    f32x4 acc[8][8];
#pragma unroll
    for (int mi = 0; mi < 8; ++mi)
#pragma unroll
        for (int ni = 0; ni < 8; ++ni)
#pragma unroll
            for (int i = 0; i < 4; ++i)
                acc[mi][ni][i] = 0.f;

    // MFMA order is row-major throughout: the first operand stays the same for 8 MFMAs in a row,
    // which this shape rewards with markedly lower power than changing both operands every time.
    //
    // First half of a step: rows 0..63.  The row fragments of the second half are fetched behind the first
    // four MFMAs, then the loads for the step NSTAGE-1 ahead (into the stage consumed in the previous step)
    // issue one every THREE MFMAs, and four MFMAs follow the last load.  The four waves of a workgroup run this
    // code in step, so their loads reach the compute unit's address unit four at a time: one every two MFMAs
    // (as first built) kept its command queue full (SQ_VMEM_TA_CMD_FIFO_FULL twenty times higher) and cost
    // 3.7 % more cycles; a load straight before the barrier stalls where nothing covers it.
#define EGTP_HALF0(fb)                                                                                 \
    {                                                                                                  \
        const unsigned char *sA = smem + cstage * STAGE_BYTES;                                         \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                  \
            fa1[i] = *(const bf16x8 *)(sA + fragA + (4 + i) * FRAG_STRIDE);                            \
        issue_loads(lvt, lkt, ldstage);                                                                \
        advance_ld();                                                                                  \
        ldstage = ldstage + 1 == NSTAGE ? 0 : ldstage + 1;                                             \
        _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                               \
            _Pragma("unroll") for (int ni = 0; ni < 8; ++ni)                                           \
                acc[mi][ni] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa0[mi], fb[ni], acc[mi][ni], 0, 0, 0); \
        _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                \
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);                                       \
            __builtin_amdgcn_sched_group_barrier(SG_DS_READ, 1, 0);                                    \
        }                                                                                              \
        _Pragma("unroll") for (int j = 0; j < 8; ++j) {                                                \
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 3, 0);                                       \
            __builtin_amdgcn_sched_group_barrier(SG_VMEM_READ, 1, 0);                                  \
        }                                                                                              \
        __builtin_amdgcn_sched_group_barrier(SG_MFMA, 4, 0);                                           \
        __builtin_amdgcn_sched_barrier(0);                                                             \
    }
    // The next step's blocks have landed (own loads; the newest NSTAGE-2 steps may still be in
    // flight) and this wave's reads of the current stage have returned; then everyone's.  After the
    // barrier the current stage may be overwritten.  A bare barrier: a fence would drain the ring.
#define EGTP_STEP_BARRIER()                                                                            \
    {                                                                                                  \
        wait_vmcnt<(NSTAGE - 2) * LOADS_PER_STEP>();                                                   \
        __builtin_amdgcn_s_waitcnt(0xC07F); /* lgkmcnt(0), the other counters unconstrained */         \
        __builtin_amdgcn_s_barrier();                                                                  \
        __builtin_amdgcn_sched_barrier(0);                                                             \
    }
    // Second half: rows 64..127.  The next step's fragments come from the next stage: rows 0..63
    // into their own registers (free by now), the column fragments into the other set; the twelve
    // reads go out behind the first twelve MFMAs, so that the last has twenty MFMAs to land.
#define EGTP_HALF1(fb, fbn)                                                                                 \
    {                                                                                                  \
        const int nstage = cstage + 1 == NSTAGE ? 0 : cstage + 1;                                      \
        const unsigned char *sN = smem + nstage * STAGE_BYTES;                                         \
        _Pragma("unroll") for (int i = 0; i < 4; ++i)                                                  \
            fa0[i] = *(const bf16x8 *)(sN + fragA + i * FRAG_STRIDE);                                  \
        _Pragma("unroll") for (int ni = 0; ni < 8; ++ni)                                               \
            fbn[ni] = *(const bf16x8 *)(sN + fragB + ni * FRAG_STRIDE);                                \
        _Pragma("unroll") for (int mi = 0; mi < 4; ++mi)                                               \
            _Pragma("unroll") for (int ni = 0; ni < 8; ++ni)                                           \
                acc[4 + mi][ni] =                                                                      \
                    __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa1[mi], fb[ni], acc[4 + mi][ni], 0, 0, 0); \
        _Pragma("unroll") for (int j = 0; j < 12; ++j) {                                               \
            __builtin_amdgcn_sched_group_barrier(SG_MFMA, 1, 0);                                       \
            __builtin_amdgcn_sched_group_barrier(SG_DS_READ, 1, 0);                                    \
        }                                                                                              \
        __builtin_amdgcn_sched_group_barrier(SG_MFMA, 20, 0);                                          \
        __builtin_amdgcn_sched_barrier(0);                                                             \
        cstage = nstage;                                                                               \
    }

    // The loop body is rotated by half a step -- [barrier, second half of step s, first half of
    // step s+1] -- so that the fragments fetched last (the column fragments) have a whole half
    // step to land before the back edge, where the compiler's wait is a conservative one.
    EGTP_HALF0(fbA);
    for (int vt = vt_begin; vt < vt_end; ++vt) {
        // two steps per trip: the column fragment sets swap roles every step (KT is even)
        for (int kt = 0; kt + 2 < KT; kt += 2) {
            EGTP_STEP_BARRIER();
            EGTP_HALF1(fbA, fbB);
            EGTP_HALF0(fbB);
            EGTP_STEP_BARRIER();
            EGTP_HALF1(fbB, fbA);
            EGTP_HALF0(fbA);
        }
        EGTP_STEP_BARRIER();
        EGTP_HALF1(fbA, fbB);
        EGTP_HALF0(fbB);
        EGTP_STEP_BARRIER();
        EGTP_HALF1(fbB, fbA);

        // pacing point: count in now, look at the counter after the fold (the round trip to the
        // L2 is hidden behind it)
        const int tiles_done = vt - vt_begin + 1;
        const bool pace_now = pace_cnt != nullptr && tiles_done % PACE_TILES == 0 && tiles_done < tps;
        if (pace_now)
            __hip_atomic_fetch_add(pace_cnt, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        // a full tile of logits is in registers: fold it into the statistics and forget it
        const int row_base = vt * BM + wm * 128 + 4 * kq;
        const bool masked = vt * BM + BM > V;
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) {
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                float z[16];
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        z[4 * q + i] = acc[4 * h + q][ni][i];
                        acc[4 * h + q][ni][i] = 0.f;
                    }
                if (masked)
                    fold16<true>(z, st[ni], row_base + h * 64, V);
                else
                    fold16<false>(z, st[ni], row_base + h * 64, V);
            }
        }
        if (pace_now) {
            // the other waves wait for this thread at the next step barrier
            const int want = pace_members * (tiles_done / PACE_TILES);
            bool met = false;
            for (int spin = 0; spin < PACE_SPINS && !met; ++spin) {
                met = __hip_atomic_load(pace_cnt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >= want;
                if (!met)
                    __builtin_amdgcn_s_sleep(PACE_SLEEP);
            }
            if (!met) {
                // the cohort is not running together: count in for every later point and stop
                const int later = (tps - 1) / PACE_TILES - tiles_done / PACE_TILES;
                if (later > 0)
                    __hip_atomic_fetch_add(pace_cnt, later, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                pace_cnt = nullptr;
            }
        }
        if (vt + 1 < vt_end)
            EGTP_HALF0(fbA);  // first half of the next tile's first step
    }
#undef EGTP_HALF0
#undef EGTP_HALF1
#undef EGTP_STEP_BARRIER

    if (pace_cnt != nullptr) {
        // a range with fewer tiles than the others leaves early: count in for the points it skips
        const int mine = vt_end - vt_begin;
        const int skipped = (tps - 1) / PACE_TILES - (mine < tps ? mine / PACE_TILES : (tps - 1) / PACE_TILES);
        if (skipped > 0)
            __hip_atomic_fetch_add(pace_cnt, skipped, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    wait_vmcnt<0>();
    __syncthreads();

    // ---- combine the four lanes, then the two waves, that hold the same token -------------
#pragma unroll
    for (int ni = 0; ni < 8; ++ni) {
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            Stats o;
            o.m = __shfl_xor(st[ni].m, off);
            o.S = __shfl_xor(st[ni].S, off);
            o.U = __shfl_xor(st[ni].U, off);
            st[ni] = merge(st[ni], o);
        }
    }
    float *red = (float *)smem;  // [wn][ni][16][3]
    if (wm == 1 && lane < 16) {
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) {
            float *r = red + ((wn * 8 + ni) * 16 + lane) * 3;
            r[0] = st[ni].m;
            r[1] = st[ni].S;
            r[2] = st[ni].U;
        }
    }
    __syncthreads();
    if (wm == 0 && lane < 16) {
        const long plane = (long)nsplit * T;
#pragma unroll
        for (int ni = 0; ni < 8; ++ni) {
            const float *r = red + ((wn * 8 + ni) * 16 + lane) * 3;
            Stats o;
            o.m = r[0];
            o.S = r[1];
            o.U = r[2];
            Stats f = merge(st[ni], o);
            const long tok = tok0 + wn * 128 + ni * 16 + lane;
            if (tok < T) {
                const long idx = (long)sp * T + tok;
                part[idx] = f.m;
                part[plane + idx] = f.S;
                part[2 * plane + idx] = f.U;
            }
        }
    }
}

}  // namespace

hipError_t k1_entropy_bf16(const void *hidden_packed, const void *w_packed, int64_t T, int K, int V,
                           const K1Plan &p, float *part, int *pace, hipStream_t st)
{
    constexpr int NSTAGE = 4;
    constexpr int LDS_BYTES = NSTAGE * STAGE_BYTES;
    static DeviceMask lds_limit_raised{0};
    hipError_t ea = raise_dynamic_lds_limit((const void *)k1_entropy_bf16_kernel<NSTAGE>, LDS_BYTES, lds_limit_raised);
    if (ea != hipSuccess)
        return ea;
    if (p.tb_tokens != BN || p.tile_v != BM || T <= 0)
        return hipErrorInvalidValue;
    const long units = (long)p.ntb * p.nsplit;
    if (units <= 0 || units > 0x7fffffffL)
        return hipErrorInvalidValue;
    const int kt = k_steps(K);
    if ((long)kt * TILE_BYTES > 0x7fffffffL)
        return hipErrorInvalidValue;  // a row tile over all of K is addressed with 32-bit byte offsets
    // pacing counters: one per cohort, cleared by a kernel (a caller may be capturing a graph)
    if (!k1_plan_paces(p))
        pace = nullptr;  // no pacing point inside a range
    if (pace != nullptr) {
        const int n = XCDS * k1_pace_cohorts(units);
        hipLaunchKernelGGL(k1_pace_zero_kernel, dim3((n + 255) / 256), dim3(256), 0, st, pace, n);
    }
    hipLaunchKernelGGL((k1_entropy_bf16_kernel<NSTAGE>), dim3((unsigned)units), dim3(256), LDS_BYTES, st,
                       (const unsigned char *)w_packed, (const unsigned char *)hidden_packed, (long)T, kt, V,
                       p.ntb, p.nsplit, p.tiles_per_split, p.ntiles_v, part, pace);
    return hipGetLastError();
}

}  // namespace egtp
