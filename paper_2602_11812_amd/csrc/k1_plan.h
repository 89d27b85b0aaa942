// Launch geometry of the fused LM-head + entropy kernels (Eq. 2).  Plain host arithmetic with no
// dependency on the HIP runtime, so that it can also be compiled and checked on its own.
#pragma once
#include <stddef.h>
#include <stdint.h>

#ifdef __HIPCC__
#define EGTP_HOST_DEVICE __host__ __device__
#else
#define EGTP_HOST_DEVICE
#endif

namespace egtp {

// Storage types of hidden states / weights (values match the public enum).
enum : int { DT_F32 = 0, DT_BF16 = 1 };

// The fused kernel contracts bf16 operands on the matrix cores.  fp32 operands reach it as sums of three bf16
// pieces each (8 + 8 + 8 significant bits: exact), and the six products of pieces that matter at fp32
// precision are laid side by side along K: a contraction six times as long over segments of d rounded up to
// whole 32-element blocks.
constexpr int K1_SPLIT_TERMS = 6;
EGTP_HOST_DEVICE inline int k1_split_segment(int d) { return (d + 31) / 32 * 32; }
EGTP_HOST_DEVICE inline long k1_contraction_len(int dtype, int d)
{
    return dtype == DT_BF16 ? (long)d : (long)K1_SPLIT_TERMS * k1_split_segment(d);
}
// largest contraction length the fused kernel addresses (32-bit byte offsets inside a packed row tile)
constexpr long K1_MAX_CONTRACTION = 4194240;

// Geometry of the fused LM-head + entropy kernel: tokens are cut into blocks of `tb_tokens`,
// the vocabulary into `nsplit` ranges of `tiles_per_split` tiles of `tile_v` rows; each
// (token block, vocabulary range) pair is one workgroup and leaves one partial (m, S, U)
// triple per token.
struct K1Plan {
    int tb_tokens;        // tokens per block
    int tile_v;           // vocabulary rows per tile
    int ntb;              // token blocks
    int ntiles_v;         // vocabulary tiles in total
    int nsplit;           // vocabulary ranges
    int tiles_per_split;  // tiles per range (last range may hold fewer)
};

K1Plan k1_plan(int dtype, int64_t T, int d, int V);
// floats needed for the partial triples of a plan (3 * nsplit * T)
size_t k1_partial_floats(const K1Plan &p, int64_t T);
// upper bound of k1_partial_floats over every T' <= T, whatever the shapes
size_t k1_partial_floats_bound(int64_t T);
// The kernel paces the workgroups that share an XCD with one counter per cohort of 32:
// cohorts per XCD for a grid of `units` workgroups, and ints to reserve for every T' <= T.
EGTP_HOST_DEVICE inline int k1_pace_cohorts(long units) { return (int)(((units + 7) / 8 + 31) / 32); }
size_t k1_pace_ints_bound(int64_t T);

// A range has a pacing point after every K1_PACE_TILES vocabulary tiles, so only
// ranges longer than that pace at all.
constexpr int K1_PACE_TILES = 4;
// Pacing serves the token blocks that share vocabulary tiles in an XCD's L2 (groups of eight): a batch of
// fewer blocks streams W_lm once from HBM whatever the workgroups' relative progress.
inline bool k1_plan_paces(const K1Plan &p) { return p.tiles_per_split > K1_PACE_TILES && p.ntb >= 8; }

}  // namespace egtp
