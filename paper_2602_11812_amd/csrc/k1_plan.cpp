// Launch geometry of the fused LM-head + entropy kernels (Eq. 2): how a batch of T tokens and a
// vocabulary of V rows is cut into (token block, vocabulary range) workgroups.  Host code only.
#include "k1_plan.h"

namespace egtp {

// ---- geometry of the fused entropy kernel ------------------------------------------------
static constexpr int TB = 256, TV = 256, TARGET_UNITS = 8192;

// compute units of the device the work is spread over (MI355X)
static constexpr int NUM_CUS = 256;
static constexpr int NSPLIT_SLACK = 8;  // how far above the minimum the number of ranges may go

K1Plan k1_plan(int dtype, int64_t T, int d, int V)
{
    K1Plan p;
    p.tb_tokens = TB;
    p.tile_v = TV;
    const int target = TARGET_UNITS;
    const long dk = k1_contraction_len(dtype, d);  // what a K sweep runs over
    p.ntb = (int)((T + p.tb_tokens - 1) / p.tb_tokens);
    p.ntiles_v = (V + p.tile_v - 1) / p.tile_v;
    int ns0 = p.ntb > 0 ? (target + p.ntb - 1) / p.ntb : 1;
    if (ns0 < 1)
        ns0 = 1;
    p.nsplit = 1;
    p.tiles_per_split = p.ntiles_v;
    if (ns0 >= p.ntiles_v) {
        // A small batch: even one range per vocabulary tile gives fewer workgroups than asked for.  What
        // counts then is the number of rounds the compute units need and what every workgroup pays to
        // start and finish (filling the load ring, the final merge and stores: about START_STEPS K steps
        // of a sweep of 2 ceil(K / 64) steps per tile).  512 tokens against 594 tiles are 1188 single-tile
        // workgroups = 5 rounds of starts, or 238 workgroups of 5 tiles each = one round of the same length.
        constexpr double START_STEPS = 6.0;
        const double start_tiles = START_STEPS / (2.0 * (double)((dk + 63) / 64));
        double best_cost = 0.0;
        for (int tps = 1; tps <= p.ntiles_v && tps <= 64; ++tps) {
            const int nsplit = (p.ntiles_v + tps - 1) / tps;
            const long units = (long)p.ntb * nsplit;
            const long rounds = (units + NUM_CUS - 1) / NUM_CUS;
            const double cost = (double)rounds * ((double)tps + start_tiles);
            if (tps == 1 || cost < best_cost - 1e-9) {
                best_cost = cost;
                p.nsplit = nsplit;
                p.tiles_per_split = tps;
            }
        }
        return p;
    }
    // One workgroup per (token block, vocabulary range), one workgroup per compute unit at a
    // time, all of about the same length: among the next few range counts take the one whose
    // last round of workgroups is fullest.
    double best = -1.0;
    for (int ns = ns0; ns <= ns0 + NSPLIT_SLACK; ++ns) {
        const int nsc = ns > p.ntiles_v ? p.ntiles_v : ns;
        const int tps = (p.ntiles_v + nsc - 1) / nsc;
        const int nsplit = (p.ntiles_v + tps - 1) / tps;
        const long units = (long)p.ntb * nsplit;
        const long rounds = (units + NUM_CUS - 1) / NUM_CUS;
        // time ~ rounds * tiles per range; work = ntb * ntiles_v tile sweeps on NUM_CUS units
        const double fill = rounds > 0 ? (double)p.ntb * p.ntiles_v / ((double)rounds * tps * NUM_CUS) : 0.0;
        if (fill > best + 1e-9) {
            best = fill;
            p.nsplit = nsplit;
            p.tiles_per_split = tps;
        }
        if (nsc == p.ntiles_v)
            break;
    }
    return p;
}

size_t k1_partial_floats(const K1Plan &p, int64_t T) { return (size_t)3 * (size_t)p.nsplit * (size_t)T; }

size_t k1_partial_floats_bound(int64_t T)
{
    // nsplit(T') <= target / ntb(T') + 1 + NSPLIT_SLACK, so
    // nsplit(T') * T' <= (target + (1 + NSPLIT_SLACK) * ntb(T')) * tb_tokens for every T' <= T
    const int64_t tbk = TB;
    const int64_t target = TARGET_UNITS;
    const int64_t ntb = (T + tbk - 1) / tbk;
    return (size_t)3 * (size_t)((target + (1 + NSPLIT_SLACK) * ntb) * tbk);
}

size_t k1_pace_ints_bound(int64_t T)
{
    // units(T') = ntb(T') * nsplit(T') <= target + (1 + NSPLIT_SLACK) * ntb(T)
    const int64_t tbk = TB;
    const int64_t target = TARGET_UNITS;
    const int64_t ntb = (T + tbk - 1) / tbk;
    return (size_t)8 * (size_t)k1_pace_cohorts((long)(target + (1 + NSPLIT_SLACK) * ntb));
}

}  // namespace egtp
