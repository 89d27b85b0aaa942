// Pieces shared by the bf16 fused entropy kernel and the kernels around it (operand packing,
// merge of the partial statistics): geometry of a packed block and the merge law of Eq. 2's
// streaming statistics.  Device-side header; no host state.
#pragma once
#include "kernels.h"

namespace egtp {
namespace {

constexpr int BK = K1_PACK_K;  // K elements per step (32)
constexpr int ROW_BYTES = BK * 2;
constexpr int TILE_BYTES = 256 * ROW_BYTES;  // one operand block, 16 KiB
constexpr float NEG_BIG = -1.0e30f;
constexpr float LOG2E = 1.4426950408889634f;
static_assert(BK == 32 && TILE_BYTES == K1_PACK_BLOCK_BYTES, "packed block geometry");

// Streaming statistics of a set of logits z against a reference m kept in log2 units (m = max z * log2 e,
// rounded once; any reference not far below the true maximum serves):
//   S = sum 2^(z log2 e - m),   U = sum 2^(z log2 e - m) (z log2 e - m);   H = ln S - U ln 2 / S.
struct Stats {
    float m, S, U;
};

// K steps of a sweep over d: K is zero-padded to a multiple of two steps, so that the main loop
// can be unrolled by two (the fragment registers swap roles every step).
__host__ __device__ __forceinline__ int k_steps(int d) { return 2 * ((d + 2 * BK - 1) / (2 * BK)); }

// XOR key of a row's four 16-byte chunks inside a packed block (64-byte rows).  With the
// fused kernel's fragment layout (lane l reads row l%16 + 16t, chunk l/16) this key makes the 16-byte-per-
// lane LDS reads as fast as a linear read; found by timing candidate keys on the hardware (most
// others, the identity included, cost a third more LDS cycles per read).
__host__ __device__ __forceinline__ int swizzle_key(int row) { return (row >> 1) & 3; }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// (m1,S1,U1) (+) (m2,S2,U2): statistics of the union of two disjoint sets of logits
__device__ __forceinline__ Stats merge(Stats a, Stats b)
{
    float M = fmaxf(a.m, b.m);
    float da = a.m - M, db = b.m - M;  // references are in log2 units already
    float sa = fast_exp2(da), sb = fast_exp2(db);
    Stats r;
    r.m = M;
    r.S = a.S * sa + b.S * sb;
    r.U = (a.U + da * a.S) * sa + (b.U + db * b.S) * sb;
    return r;
}

}  // namespace
}  // namespace egtp
