// Prediction head (Section 3.2): pooled vector -> perceptron d -> d_h (ReLU) -> n_out, then
// either the scalar itself (n_out == 1) or the expected value over K bins of Eq. 6.
//
// Layer 1 is a small [B x d] . [d x d_h] contraction kept entirely in fp32 (the pooled
// vector is never re-rounded); the plain kernel is LDS-tiled, 64 x 64 outputs per workgroup, 4 x 4
// per thread.  The contraction is split along d so that about a thousand workgroups exist even for one
// small batch; the splits leave partial pre-activations that layer 2 adds in split order
// (fixed order, bit-reproducible) before bias and ReLU.  Layer 2 and the K-bin decode are one
// workgroup per sequence.
//
// With bf16 weights and d a multiple of 8, layer 1 runs on the bf16 matrix cores without
// rounding the pooled vector: an fp32 value is the exact sum of three bf16 values (its top 8
// significant bits, the top 8 of what is left, and the rest), a bf16 x bf16 product is exact in
// fp32, so three MFMAs per weight fragment accumulate the same products an fp32 dot product
// would, in fp32.  Fragments come straight from global memory: a lane's 8 K-elements are 16
// contiguous bytes of a weight row and 32 contiguous bytes of a pooled row.
#include "bf16_split.h"
#include "kernels.h"
#include "partial_planes.h"
#include "wave_reduce.h"

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

// Layer 1 for at most SK_SEQS sequences and fp32 weights (a training batch, a handful of requests): the work is
// one pass over W1, so the kernel is built around streaming it.  Workgroup = 16 head rows x one slice of at most
// SK_SLICE elements of d; the slice of all pooled vectors sits in LDS (zero rows for missing sequences).  A wave
// owns 4 rows; lane l takes K elements 4l .. 4l+3 of every 256: one 16-byte load per row, sixteen 16-byte LDS
// reads, 256 FMAs into 4 x 16 accumulators.  The 64 accumulators are then summed over the 64 lanes by a halving
// butterfly (a lane passes on the half it does not keep: 63 exchanges instead of 384), which leaves lane l with
// the total of (row l / 16, sequence l % 16).  Fixed order: bit-reproducible.
constexpr int SK_SEQS = 16, SK_SLICE = 512, SK_ROWS = 16;

__global__ __launch_bounds__(256) void head_layer1_skinny_kernel(const float *__restrict__ x,
                                                                 const int32_t *__restrict__ slot, int B, int d,
                                                                 int d_h, const float *__restrict__ w1, int kchunk,
                                                                 float *__restrict__ act_part)
{
    __shared__ __align__(16) float xs[SK_SEQS][SK_SLICE];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int kbeg = blockIdx.y * kchunk;
    const int klen = min(d - kbeg, kchunk);  // a multiple of 4; <= 0 past the end of d: the plane is zeros
    // lane b learns the state row of sequence b (asked for first: the counter of outstanding loads is in order)
    int my_row = lane < B ? lane : 0;
    if (slot)
        my_row = slot[my_row];
    // this lane's share of W1 next -- all of it in flight at once: a load per pass would be as many HBM
    // latencies in a row
    const int j0 = blockIdx.x * SK_ROWS + wave * 4;
    constexpr int PASSES = SK_SLICE / 256;
    float4 wv[PASSES][4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int j = j0 + r < d_h ? j0 + r : d_h - 1;  // clamped rows are computed and dropped
        const float *wrow = w1 + (long)j * d + (klen > 0 ? kbeg : 0);
#pragma unroll
        for (int p = 0; p < PASSES; ++p) {
            // pieces past the end of the slice: load piece 0 instead (no branch around a load, so that the
            // loads stay countable and the waits below can be exact); the staged vectors are zero there
            const int k = 4 * lane + 256 * p;
            wv[p][r] = *(const float4 *)(wrow + (k < klen ? k : 0));
        }
    }
    // meanwhile stage the slice of the pooled vectors, every thread the same 16-byte piece of several rows.  All
    // its loads are issued before the first store (addresses are clamped, not branched on: a wait per row
    // would be sixteen cache latencies in a row); rows and pieces that do not exist become zeros.
    constexpr int PIECES = SK_SLICE / 4;      // 16-byte pieces per staged row
    constexpr int ROWS_AT_ONCE = 256 / PIECES;  // rows the 256 threads cover in one go
    static_assert(256 % PIECES == 0 && PIECES % 64 == 0 && SK_SEQS % ROWS_AT_ONCE == 0, "staging layout");
    const int pc = tid % PIECES;
    const int brow = __builtin_amdgcn_readfirstlane(tid / PIECES);  // the same for a whole wave
    const bool piece_ok = 4 * pc < klen;
    const long piece = piece_ok ? (long)kbeg + 4 * pc : 0;
    float4 xv16[SK_SEQS / ROWS_AT_ONCE];
#pragma unroll
    for (int i = 0; i < SK_SEQS / ROWS_AT_ONCE; ++i) {
        // sequences past B read the row of sequence 0 (lane b of my_row holds 0 for them)
        const long xrow = __builtin_amdgcn_readlane(my_row, brow + ROWS_AT_ONCE * i);
        xv16[i] = *(const float4 *)(x + xrow * (long)d + piece);
    }
#pragma unroll
    for (int i = 0; i < SK_SEQS / ROWS_AT_ONCE; ++i) {
        const int b = brow + ROWS_AT_ONCE * i;
        const bool ok = piece_ok && b < B;
        float4 v = xv16[i];
        v.x = ok ? v.x : 0.f, v.y = ok ? v.y : 0.f, v.z = ok ? v.z : 0.f, v.w = ok ? v.w : 0.f;
        *(float4 *)&xs[b][4 * pc] = v;
    }
    __syncthreads();

    float acc[64];  // acc[16 * r + b]
#pragma unroll
    for (int i = 0; i < 64; ++i)
        acc[i] = 0.f;
#pragma unroll
    for (int p = 0; p < PASSES; ++p) {
        const int k = 4 * lane + 256 * p;  // past klen: the staged vectors are zero
#pragma unroll
        for (int b = 0; b < SK_SEQS; ++b) {
            const float4 xv = *(const float4 *)&xs[b][k];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                float a = acc[16 * r + b];
                a = fmaf(wv[p][r].x, xv.x, a);
                a = fmaf(wv[p][r].y, xv.y, a);
                a = fmaf(wv[p][r].z, xv.z, a);
                a = fmaf(wv[p][r].w, xv.w, a);
                acc[16 * r + b] = a;
            }
        }
    }
    // halving butterfly over the lanes: after the step with distance o a lane holds n / 2 sums, the upper half
    // of the indices if its bit o is set
#pragma unroll
    for (int o = 32, n = 64; o >= 1; o >>= 1, n >>= 1) {
        const bool upper = (lane & o) != 0;
#pragma unroll
        for (int i = 0; i < n / 2; ++i) {
            const float keep = upper ? acc[i + n / 2] : acc[i];
            const float pass = upper ? acc[i] : acc[i + n / 2];
            acc[i] = keep + __shfl_xor(pass, o);
        }
    }
    const int b = lane & 15, j = j0 + (lane >> 4);
    if (b < B && j < d_h)
        act_part[((long)blockIdx.y * B + b) * d_h + j] = acc[0];
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int MK = 32;  // K elements per MFMA step

// 8 fp32 values -> three bf16 fragments whose sum is exactly the input (truncating splits)
__device__ __forceinline__ void split3(const float (&f)[8], bf16x8 &hi, bf16x8 &mid, bf16x8 &lo)
{
    unsigned h[8], m[8], l[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        split3_bits(f[i], h[i], m[i], l[i]);
    }
    u32x4 ph, pm, pl;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        ph[i] = (h[2 * i] >> 16) | h[2 * i + 1];
        pm[i] = (m[2 * i] >> 16) | m[2 * i + 1];
        pl[i] = (l[2 * i] >> 16) | l[2 * i + 1];
    }
    hi = __builtin_bit_cast(bf16x8, ph);
    mid = __builtin_bit_cast(bf16x8, pm);
    lo = __builtin_bit_cast(bf16x8, pl);
}

// Layer 1 on the matrix cores, bf16 weights, d % 8 == 0.  Workgroup = 4 waves, MJ = 128 head rows x
// TN = 64 sequences; wave = 64 x 32 = 4 x 2 MFMA 16x16x32 tiles, weights as the row operand (lane l:
// head row l % 16, K elements 8 * (l / 16) .. + 8), pooled vectors as the column operand; in the
// accumulator a lane holds head rows 4 * (l / 16) + i of sequence l % 16.  Per K step every thread
// fetches 8 K-elements of one pooled row (32 bytes) and of two weight rows (16 bytes each), splits
// the fp32 values once, and leaves all of it in LDS in fragment order -- fragment f, lane l at
// (f * 64 + l) * 16 bytes -- so that a fragment read is one linear 16-byte read per lane.  Two
// LDS buffers; global fetches run three steps ahead in registers.
constexpr int MJ = 128;
constexpr int MFMA_W_FRAGS = MJ / 16;             // 8 weight fragments per step
constexpr int MFMA_X_FRAGS = 3 * (TN / 16);       // 3 parts x 4 sequence fragments
constexpr int MFMA_STAGE_BYTES = (MFMA_W_FRAGS + MFMA_X_FRAGS) * 1024;

__global__ __launch_bounds__(256) void head_layer1_mfma_kernel(const float *__restrict__ x,
                                                               const int32_t *__restrict__ slot, int B, int d,
                                                               int d_h, const unsigned short *__restrict__ w1,
                                                               int kchunk, int nks, int jtiles,
                                                               float *__restrict__ act_part)
{
    __shared__ __align__(16) unsigned char lds[2 * MFMA_STAGE_BYTES];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int l15 = lane & 15, kq = lane >> 4;
    // Workgroup i runs on XCD i % 8: the slice along d varies fastest, so that an XCD's L2 only
    // ever pulls its own slices of the weights and of the pooled vectors over the fabric.
    const int kslice = blockIdx.x % nks;
    const int tile = blockIdx.x / nks;
    const int j0 = (tile % jtiles) * MJ, s0 = (tile / jtiles) * TN;
    const int wj = (wave & 1) * 4;  // first of this wave's 4 weight fragments
    const int ws = (wave >> 1) * 2; // first of its 2 sequence fragments

    // what this thread stages: row 16 * wave + lane % 16 of the tile (and that row + 64 of the
    // weights), K elements 8 * (lane / 16) .. + 8 -- which is lane `lane` of fragment `wave`, so a
    // wave's 16-byte LDS writes are one linear KiB
    const int srow_l = wave * 16 + l15, kpart = kq;
    int srow = s0 + srow_l;
    srow = srow < B ? srow : B - 1;  // clamped rows are computed and dropped
    const long xrow = slot ? slot[srow] : srow;
    const float *xp = x + xrow * (long)d + 8 * kpart;
    const unsigned short *wp[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        int jrow = j0 + 64 * r + srow_l;
        jrow = jrow < d_h ? jrow : d_h - 1;
        wp[r] = w1 + (long)jrow * d + 8 * kpart;
    }
    const unsigned stage_lane = (unsigned)(lane * 16);
    const unsigned w_dst0 = (unsigned)(wave * 1024) + stage_lane;                   // rows 0..63
    const unsigned w_dst1 = (unsigned)((4 + wave) * 1024) + stage_lane;             // rows 64..127
    const unsigned x_dst = (unsigned)((MFMA_W_FRAGS + wave) * 1024) + stage_lane;   // part p: + p * 4096

    f32x4 acc[4][2];
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
            acc[a][b] = f32x4{0.f, 0.f, 0.f, 0.f};

    const int kbeg = kslice * kchunk;
    const int kend = min(d, kbeg + kchunk);
    // kend and 8 * kpart are multiples of 8: a thread's 8 elements are inside [kbeg, kend) or all outside
    struct Fetched {
        u32x4 w[2];
        float4 x[2];
    };
    auto fetch = [&](int k0, Fetched &r) {
        r.w[0] = r.w[1] = u32x4{0u, 0u, 0u, 0u};
        r.x[0] = r.x[1] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (k0 + 8 * kpart < kend) {
            r.w[0] = *(const u32x4 *)(wp[0] + k0);
            r.w[1] = *(const u32x4 *)(wp[1] + k0);
            r.x[0] = *(const float4 *)(xp + k0);
            r.x[1] = *(const float4 *)(xp + k0 + 4);
        }
    };
    auto stage = [&](const Fetched &r, unsigned char *buf) {
        const float f[8] = {r.x[0].x, r.x[0].y, r.x[0].z, r.x[0].w, r.x[1].x, r.x[1].y, r.x[1].z, r.x[1].w};
        bf16x8 hi, mid, lo;
        split3(f, hi, mid, lo);
        *(u32x4 *)(buf + w_dst0) = r.w[0];
        *(u32x4 *)(buf + w_dst1) = r.w[1];
        *(bf16x8 *)(buf + x_dst) = hi;
        *(bf16x8 *)(buf + x_dst + 4096) = mid;
        *(bf16x8 *)(buf + x_dst + 8192) = lo;
    };

    // Operands are fetched three steps ahead into a ring of three register sets (the loop is
    // unrolled by three so that the ring is indexed statically) and staged one step ahead.
    Fetched ring[3];
    fetch(kbeg, ring[0]);
    fetch(kbeg + MK, ring[1]);
    fetch(kbeg + 2 * MK, ring[2]);
    stage(ring[0], lds);
    __syncthreads();
    int cur = 0;
    for (int base = kbeg; base < kend; base += 3 * MK) {
#pragma unroll
        for (int u = 0; u < 3; ++u) {
            const int k0 = base + u * MK;
            if (k0 >= kend)
                break;
            fetch(k0 + 3 * MK, ring[u]);  // ring[u] held step k0, which is in LDS already
            const unsigned char *buf = lds + cur * MFMA_STAGE_BYTES;
            bf16x8 wf[4], xf[3][2];
#pragma unroll
            for (int a = 0; a < 4; ++a)
                wf[a] = *(const bf16x8 *)(buf + ((wj + a) * 64 + lane) * 16);
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int b = 0; b < 2; ++b)
                    xf[p][b] = *(const bf16x8 *)(buf + ((MFMA_W_FRAGS + 4 * p + ws + b) * 64 + lane) * 16);
#pragma unroll
            for (int p = 2; p >= 0; --p)  // smallest parts first
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 2; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[a], xf[p][b], acc[a][b], 0, 0, 0);
            if (k0 + MK < kend)
                stage(ring[(u + 1) % 3], lds + (cur ^ 1) * MFMA_STAGE_BYTES);  // nobody reads that buffer now
            __syncthreads();
            cur ^= 1;
        }
    }

    float *act = act_part + (long)kslice * B * d_h;
#pragma unroll
    for (int b = 0; b < 2; ++b) {
        const int s = s0 + 16 * (ws + b) + l15;
        if (s >= B)
            continue;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            const int jj = j0 + 16 * (wj + a) + 4 * kq;
            if (jj + 3 < d_h && (d_h & 3) == 0) {
                *(f32x4 *)(act + (long)s * d_h + jj) = acc[a][b];
            } else {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    if (jj + i < d_h)
                        act[(long)s * d_h + jj + i] = acc[a][b][i];
            }
        }
    }
}

// one workgroup (4 waves) per sequence: out[o] = b2[o] + w2[o,:] . act[b,:]; n_out > 1 => Eq. 6
// LDS: a[d_h] | partial[4][n_out]
template <bool WBF16>
__global__ __launch_bounds__(256) void head_layer2_kernel(const float *__restrict__ act_part, int nks, int B,
                                                          const float *__restrict__ b1, int d_h, int n_out,
                                                          const void *__restrict__ w2,
                                                          const float *__restrict__ b2,
                                                          const float *__restrict__ centers,
                                                          float *__restrict__ pred,
                                                          float *__restrict__ p_hat)
{
    const int b = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    extern __shared__ __align__(16) float a[];
    float *partial = a + d_h;
    // hidden activations: partial sums in split order, then bias and ReLU; kept in LDS
    if ((d_h & 3) == 0) {
        for (int j = tid * 4; j < d_h; j += 1024) {
            const float4 pre = sum_planes4(act_part, nks, B, b, d_h, j);
            const float v[4] = {pre.x, pre.y, pre.z, pre.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const float p = v[i] + (b1 ? b1[j + i] : 0.f);
                a[j + i] = p > 0.f ? p : 0.f;
            }
        }
    } else {
        for (int j = tid; j < d_h; j += 256) {
            float pre = 0.f;
#pragma unroll 8
            for (int z = 0; z < nks; ++z)
                pre += act_part[((long)z * B + b) * d_h + j];
            pre += b1 ? b1[j] : 0.f;
            a[j] = pre > 0.f ? pre : 0.f;
        }
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
    // the distribution itself (Eq. 6's p-hat), when the caller wants it: bin o by lane o % 64
    if (p_hat != nullptr && n_out > 1) {
        const float inv = 1.0f / den;
        for (int o = lane; o < n_out; o += 64) {
            const float s = ((partial[o] + partial[n_out + o]) + (partial[2 * n_out + o] + partial[3 * n_out + o])) +
                            (b2 ? b2[o] : 0.f);
            p_hat[(long)b * n_out + o] = __expf(s - m) * inv;
        }
    }
}

}  // namespace

// slices of the skinny kernel: as few as keep a slice within its LDS buffer
static int skinny_slices(int d) { return (d + SK_SLICE - 1) / SK_SLICE; }
static bool skinny_serves(int d, int32_t B, int wdtype)
{
    return wdtype == DT_F32 && B <= SK_SEQS && d % 4 == 0 && skinny_slices(d) <= 64;
}

int head_k_splits(int d, int d_h, int32_t B, int wdtype)
{
    if (skinny_serves(d, B, wdtype))
        return skinny_slices(d);
    int base = (d + 511) / 512;  // slices of at most 512 along d ...
    base = base < 1 ? 1 : (base > 8 ? 8 : base);
    const long tiles = (long)((d_h + TM - 1) / TM) * ((B + TN - 1) / TN);
    long want = tiles > 0 ? (1024 + tiles - 1) / tiles : 1;  // ... thinner when the batch has few tiles
    const int cap = (d + TK - 1) / TK < 64 ? (d + TK - 1) / TK : 64;
    long n = want > base ? want : base;
    n = n > cap ? cap : n;
    return n < 1 ? 1 : (int)n;
}

size_t head_act_floats_bound(int d, int d_h, int32_t B, int wdtype)
{
    // the number of planes only depends on how many 64-sequence tiles the batch has -- and, for fp32 weights,
    // on whether the batch is small enough for the skinny kernel
    size_t best = 0;
    for (int32_t st = 1; st <= (B + TN - 1) / TN; ++st) {
        const int32_t b = st * TN < B ? st * TN : B;
        const size_t f = (size_t)head_k_splits(d, d_h, b, wdtype) * (size_t)b * (size_t)d_h;
        best = f > best ? f : best;
    }
    const int32_t bs = B < SK_SEQS ? B : SK_SEQS;
    const size_t fs = (size_t)head_k_splits(d, d_h, bs, wdtype) * (size_t)bs * (size_t)d_h;
    return fs > best ? fs : best;
}

hipError_t head_layer1(const float *x, const int32_t *slot, int32_t B, int d, int d_h, const void *w1,
                       int wdtype, float *act_part, hipStream_t st)
{
    if (B <= 0)
        return hipSuccess;
    const int nks = head_k_splits(d, d_h, B, wdtype);
    if (skinny_serves(d, B, wdtype)) {
        // whole 256-element passes; nks = ceil(d / SK_SLICE) keeps a slice within the LDS buffer and leaves no
        // slice empty (a slice past the end of d would still write its plane: zeros)
        const int kchunk_s = ((d + nks - 1) / nks + 255) / 256 * 256;
        if (kchunk_s > SK_SLICE)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL(head_layer1_skinny_kernel, dim3((d_h + SK_ROWS - 1) / SK_ROWS, nks), dim3(256), 0, st, x, slot,
                           B, d, d_h, (const float *)w1, kchunk_s, act_part);
        return hipGetLastError();
    }
    const dim3 grid((d_h + TM - 1) / TM, (B + TN - 1) / TN, nks);
    if (wdtype == DT_BF16 && d % 8 == 0) {
        // matrix-core path: slices are multiples of the MFMA K step (late slices may be empty
        // and then write zeros)
        const int kchunk_m = ((d + nks - 1) / nks + MK - 1) / MK * MK;
        const int jtiles = (d_h + MJ - 1) / MJ;
        const long wgs = (long)jtiles * ((B + TN - 1) / TN) * nks;
        if (wgs > 0x7fffffffL)
            return hipErrorInvalidValue;
        hipLaunchKernelGGL(head_layer1_mfma_kernel, dim3((unsigned)wgs), dim3(256), 0, st, x, slot, B, d, d_h,
                           (const unsigned short *)w1, kchunk_m, nks, jtiles, act_part);
        return hipGetLastError();
    }
    const int kchunk = ((d + nks - 1) / nks + TK - 1) / TK * TK;  // multiple of the K step
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
    const int nks = head_k_splits(a.d, a.d_h, a.B, a.wdtype);
    const size_t lds2 = ((size_t)a.d_h + 4 * (size_t)a.n_out) * sizeof(float);
    if (lds2 > 96 * 1024)
        return hipErrorInvalidValue;
    static DeviceMask raised_bf16{0}, raised_f32{0};
    hipError_t e1 = raise_dynamic_lds_limit((const void *)head_layer2_kernel<true>, 96 * 1024, raised_bf16);
    hipError_t e2 = raise_dynamic_lds_limit((const void *)head_layer2_kernel<false>, 96 * 1024, raised_f32);
    if (e1 != hipSuccess || e2 != hipSuccess)
        return e1 != hipSuccess ? e1 : e2;
    hipError_t e = head_layer1(a.x, a.slot, a.B, a.d, a.d_h, a.w1, a.wdtype, a.act, st);
    if (e != hipSuccess)
        return e;
    if (a.wdtype == DT_BF16)
        hipLaunchKernelGGL(head_layer2_kernel<true>, dim3(a.B), dim3(256), lds2, st, a.act, nks, a.B, a.b1, a.d_h,
                           a.n_out, a.w2, a.b2, a.bin_centers, a.pred, a.p_hat);
    else
        hipLaunchKernelGGL(head_layer2_kernel<false>, dim3(a.B), dim3(256), lds2, st, a.act, nks, a.B, a.b1, a.d_h,
                           a.n_out, a.w2, a.b2, a.bin_centers, a.pred, a.p_hat);
    return hipGetLastError();
}

}  // namespace egtp
