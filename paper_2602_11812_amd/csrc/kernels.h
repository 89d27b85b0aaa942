// Internal launcher interface between the C-ABI layer and the gfx950 kernels.
// Nothing here is exported; all pointers are device pointers unless stated otherwise.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "k1_plan.h"

namespace egtp {

// One bit per device, set once something has been done for that device.  Shared by every context
// and thread of the process, hence atomic; two first calls that race only repeat the action.
using DeviceMask = std::atomic<unsigned long long>;
inline bool device_bit_set(const DeviceMask &m, int dev)
{
    return dev >= 0 && dev < 64 && ((m.load(std::memory_order_acquire) >> dev) & 1ull);
}
inline void set_device_bit(DeviceMask &m, int dev)
{
    if (dev >= 0 && dev < 64)
        m.fetch_or(1ull << dev, std::memory_order_release);
}

// Raises a kernel's dynamic LDS limit once per device; `done` is the caller's mask of the devices
// it has been raised on.
inline hipError_t raise_dynamic_lds_limit(const void *kernel, int bytes, DeviceMask &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return e;
    if (device_bit_set(done, dev))
        return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess)
        set_device_bit(done, dev);
    return e;
}

// Packed operand layout of the matrix-core kernel: blocks of 256 rows x K1_PACK_K bf16
// elements (K1_PACK_BLOCK_BYTES each), block (row tile, K step) at index tile * steps + step with
// steps = 2 * ceil(K / (2 K1_PACK_K)) (an even number), stored in LDS-image order; rows and K zero-padded
// to whole blocks.  K is the contraction length the kernel sees: d for bf16 operands,
// k1_contraction_len(DT_F32, d) for fp32 operands split into bf16 pieces.
constexpr int K1_PACK_K = 32;
constexpr int K1_PACK_BLOCK_BYTES = 256 * K1_PACK_K * 2;
size_t k1_packed_bytes(int64_t rows, int K);
hipError_t k1_pack_rows_bf16(const void *src, int64_t rows, int d, void *dst, hipStream_t st);
// fp32 rows (d % 4 == 0) into the six K segments of the W_lm side or of the hidden-state side
hipError_t k1_pack_rows_f32_split(const void *src, int64_t rows, int d, bool hidden_side, void *dst,
                                  hipStream_t st);

// Eq. 2, fused: partial (m = max z log2 e, sum e^{z-m}, sum e^{z-m}(z-m) log2 e) per token and vocabulary range.
// Both operands in the packed layout, contraction length K; `pace`: k1_pace_ints_bound ints of scratch
// (contents do not matter on entry), or NULL to run without pacing.
hipError_t k1_entropy_bf16(const void *hidden_packed, const void *w_packed, int64_t T, int K, int V,
                           const K1Plan &p, float *part, int *pace, hipStream_t st);
// merges the nsplit partial triples of each token in a fixed order; entropy[t] = ln S - U/S
hipError_t k1_merge(const float *part, int nsplit, int64_t T, float *entropy, hipStream_t st);

// Ragged plumbing.
hipError_t scan_lengths(const int32_t *lengths, int32_t B, int32_t *offsets, hipStream_t st);
hipError_t segment_ids(const int32_t *offsets, int32_t B, int64_t T, int32_t *seg, hipStream_t st);

// Eq. 3 / Eq. 4 / Eq. 8 over ragged offsets.  A sequence is cut into units of at most
// POOL_UNIT tokens; unit_start[B+1] is the exclusive scan of units per sequence.
constexpr int POOL_UNIT = 128;
inline int64_t pool_units_bound(int64_t T, int32_t B) { return (T + POOL_UNIT - 1) / POOL_UNIT + B; }

struct PoolArgs {
    const void *hidden;       // [T x d]
    int dtype;
    int d;
    float *entropy;           // [T]; read, or -- one token per sequence with k1_part set -- written
    const float *k1_part;     // one token per sequence only: the fused kernel's partial triples, still to be
    int k1_nsplit;            //   merged into entropy (k1_nsplit ranges), or NULL = entropy is final
    const int32_t *offsets;   // [B+1], or NULL = one token per sequence
    const int32_t *slot;      // [B] or NULL
    int32_t B;
    int64_t T;
    float inv_alpha;
    const float *state_lse;   // [S] old state or NULL (= empty state)
    const float *state_pooled;// [S x d] old state or NULL
    float *out_pooled;        // [S x d] (may alias state_pooled)
    float *out_lse;           // [S]     (may alias state_lse)
    // workspace
    int32_t *unit_start;      // [B+1]
    float *lse_new;           // [B]
    float *state_scale;       // [B]
    float *partial;           // [units_bound x d]
};
hipError_t pool_entropy_weighted(const PoolArgs &a, hipStream_t st);

// Table 3 alternatives: kind 0 average, 1 max, 2 last token.  Average and max use the unit table
// (unit_start[B+1]) and the unit partials ([pool_units_bound(T, B) x d]) of the weighted pooling.
hipError_t pool_plain(const void *hidden, int dtype, int d, const int32_t *offsets, int32_t B, int64_t T,
                      int kind, int32_t *unit_start, float *partial, float *out_pooled, hipStream_t st);

// Prediction head.
struct HeadArgs {
    const float *x;           // [S x d] pooled vectors
    const int32_t *slot;      // [B] row of x per sequence, or NULL = identity
    int32_t B;
    int d, d_h, n_out, wdtype;
    const void *w1; const float *b1;
    const void *w2; const float *b2;
    const float *bin_centers; // [n_out] when n_out > 1
    float *act;               // workspace, head_act_floats_bound(d, d_h, B, wdtype) floats: partial pre-activations
    float *pred;              // [B]
    float *p_hat;             // [B x n_out] softmax over the bins (Eq. 6), or NULL; n_out > 1 only
};
// Number of partial pre-activation planes layer 1 leaves: it is split along d so that about a
// thousand workgroups exist whatever the batch (a small batch gets many thin slices); a small batch on fp32
// weights is served by a kernel of its own that leaves one plane per 512 elements of d.
int head_k_splits(int d, int d_h, int32_t B, int wdtype);
// floats of partial planes sufficient for every batch of at most B sequences
size_t head_act_floats_bound(int d, int d_h, int32_t B, int wdtype);
hipError_t head_forward(const HeadArgs &a, hipStream_t st);
// layer 1 alone: partial pre-activations act_part[head_k_splits(d, d_h, B, wdtype) x B x d_h] (no bias, no ReLU)
hipError_t head_layer1(const float *x, const int32_t *slot, int32_t B, int d, int d_h, const void *w1,
                       int wdtype, float *act_part, hipStream_t st);

// One training step of a K-bin head on frozen features (Eq. 5, 7, 9 + AdamW), fp32 parameters.
struct TrainArgs {
    const float *x;            // [B x d] features
    const int32_t *bin;        // [B] target bin
    const float *y;            // [B] target length
    const int32_t *steps;      // [B] decode steps of the sample's sequence (Eq. 9), or NULL
    int32_t n_seqs;            // sequences in the batch when steps != NULL
    int32_t B;
    int d, d_h, K;
    float *w1, *b1, *w2, *b2;  // parameters, updated in place
    float *m_w1, *v_w1, *m_b1, *v_b1, *m_w2, *v_w2, *m_b2, *v_b2;  // AdamW moments
    const float *centers;      // [K]
    float lambda, lr, beta1, beta2, eps, weight_decay;
    float omb1, omb2;          // 1 - beta1, 1 - beta2 (rounded once from double)
    float corr1, corr2;        // 1 - beta1^t, 1 - beta2^t
    float *g_w1, *g_b1, *g_w2, *g_b2;  // optional copies of the gradients
    float *loss;               // [3] total, CE part, MSE part
    // workspace
    float *act_part;           // head_act_floats_bound(d, d_h, B, DT_F32) floats
    float *act;                // [B x d_h]
    float *dact;               // [B x d_h]
    float *dz;                 // [B x K]
    float *loss_part;          // [B x 2]
};
hipError_t head_train_step(const TrainArgs &a, hipStream_t st);

// Register-only MFMA loop (measurement aid): MFMA_PROBE_WORKGROUPS workgroups of 4 waves, each
// wave `iters` steps of 64 MFMAs; sink holds one float per thread.
constexpr int MFMA_PROBE_WORKGROUPS = 1024;
double mfma_probe_flop(int iters);
hipError_t mfma_probe_launch(float *sink, int iters, int random_operands, hipStream_t st);


// Plain streaming read of a buffer (measurement aid): HBM_PROBE_WORKGROUPS workgroups, each reading one
// contiguous slab with 16-byte loads; sink holds one word per thread.
constexpr int HBM_PROBE_WORKGROUPS = 8192;
hipError_t hbm_read_probe_launch(const void *buf, size_t bytes, unsigned *sink, hipStream_t st);

}  // namespace egtp
