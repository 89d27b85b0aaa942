// Host-code checks meant to run under AddressSanitizer + UndefinedBehaviorSanitizer.
//
// Linked with the fp64 oracle (oracle/egtp_oracle.c), the scheduling model (csrc/sched.cpp) and the
// launch-plan arithmetic (csrc/k1_plan.cpp), all compiled for the host with
// -fsanitize=address,undefined.  Every exported function of the three is driven over ragged, empty
// and boundary-sized inputs in buffers of exactly the documented size, so that an index past an
// array, a signed overflow or a misaligned access ends the program; the results are checked
// against hand-derived values (Eq. 2-4 on a d = 2, V = 4 example; closed forms) and invariants.
// Exit status 0 = everything passed and no sanitizer report.  No GPU, no HIP runtime.
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

#include "../include/egtp_sched.h"
#include "../paper_2602_11812_amd/csrc/k1_plan.h"

extern "C" {
int oracle_offsets(const int32_t *lengths, int32_t B, int32_t *offsets);
int oracle_seg_ids(const int32_t *offsets, int32_t B, int64_t T, int32_t *seg);
int oracle_entropy_from_logits(const double *z, int64_t T, int32_t V, double *H);
int oracle_logits(const void *hidden_row, const void *w_lm, int dtype, int32_t d, int32_t V, double *z);
int oracle_entropy(const void *hidden, const void *w_lm, int dtype, int64_t T, int32_t d, int32_t V, double *H);
int oracle_pool(const void *hidden, int dtype, int32_t d, const double *H, const int32_t *offsets, int32_t B,
                double alpha, double *w, double *pooled, double *lse);
int oracle_pool_ablation(const void *hidden, int dtype, int32_t d, const int32_t *offsets, int32_t B, int kind,
                         double *pooled);
int oracle_head(const double *x, int32_t B, int32_t d, int32_t d_h, int32_t n_out, const void *w1, const float *b1,
                const void *w2, const float *b2, int wdtype, double *out);
int oracle_bin_decode(const double *logits, int32_t B, int32_t K, const double *centers, double *p_hat,
                      double *y_hat);
int oracle_soft_label(int32_t i, int32_t K, double *p);
int oracle_head_loss_grad(const double *x, const int32_t *bin, const double *y, const double *weight, int32_t B,
                          int32_t d, int32_t d_h, int32_t K, const double *w1, const double *b1, const double *w2,
                          const double *b2, const double *c, double lambda, double *loss3, double *g_w1,
                          double *g_b1, double *g_w2, double *g_b2);
int oracle_adamw(double *w, double *m, double *v, const double *g, int64_t n, double lr, double beta1, double beta2,
                 double eps, double weight_decay, int64_t t);
}

namespace {

int failures = 0;
#define CHECK(cond)                                                          \
    do {                                                                     \
        if (!(cond)) {                                                       \
            std::fprintf(stderr, "%s:%d: check failed: %s\n", __FILE__, __LINE__, #cond); \
            ++failures;                                                      \
        }                                                                    \
    } while (0)

bool close_to(double a, double b, double tol) { return std::fabs(a - b) <= tol * (1.0 + std::fabs(b)); }

// xorshift: the checks need arbitrary, reproducible numbers, nothing more
struct Rng {
    uint64_t s;
    explicit Rng(uint64_t seed) : s(seed * 0x9E3779B97F4A7C15ull + 1) {}
    uint64_t next()
    {
        s ^= s << 13;
        s ^= s >> 7;
        s ^= s << 17;
        return s;
    }
    double uniform() { return (double)(next() >> 11) / (double)(1ull << 53); }
    double normal() { return std::sqrt(-2.0 * std::log(uniform() + 1e-300)) * std::cos(6.283185307179586 * uniform()); }
    int below(int n) { return (int)(next() % (uint64_t)n); }
};

uint16_t to_bf16(float f)
{
    uint32_t u;
    std::memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// ---- oracle: the worked example (d = 2, V = 4), derived by hand from Eq. 2-4 and Section 3.2 ----------------
void oracle_worked_example()
{
    const double ln2 = std::log(2.0);
    const float W[8] = {(float)-ln2, 0.f, (float)(-2 * ln2), 0.f, (float)(-3 * ln2), 0.f, (float)(-3 * ln2), 0.f};
    // the fp32 rounding of ln 2 moves the entropies by ~1e-8; the bars below allow for it
    const float h[6] = {0.f, 1.f, 1.f, 2.f, 200.f, 3.f};
    double H[3];
    CHECK(oracle_entropy(h, W, 0, 3, 2, 4, H) == 0);
    CHECK(close_to(H[0], std::log(4.0), 1e-12));
    CHECK(close_to(H[1], 1.75 * ln2, 1e-7));
    CHECK(H[2] >= 0.0 && H[2] < 1e-50);
    const int32_t off[2] = {0, 3};
    double w[3], pooled[2], lse;
    CHECK(oracle_pool(h, 0, 2, H, off, 1, 1.0, w, pooled, &lse) == 0);
    CHECK(close_to(w[0], 0.478263768929, 1e-7) && close_to(w[1], 0.402170288838, 1e-7) &&
          close_to(w[2], 0.119565942232, 1e-7));
    CHECK(close_to(pooled[0], 24.315358735303, 1e-7) && close_to(pooled[1], 1.641302173303, 1e-7));
    CHECK(close_to(lse, 2.123887241962, 1e-7));
    const float w1[4] = {1.f, -1.f, 0.5f, 0.5f}, b1[2] = {0.f, -1.f}, w2[2] = {2.f, -1.f}, b2[1] = {0.5f};
    double y;
    CHECK(oracle_head(pooled, 1, 2, 2, 1, w1, b1, w2, b2, 0, &y) == 0);
    CHECK(close_to(y, 33.869782669697, 1e-7));
    // temperature 0.5 on the same three tokens
    CHECK(oracle_pool(h, 0, 2, H, off, 1, 0.5, w, pooled, &lse) == 0);
    CHECK(close_to(w[0], 0.565097292026, 1e-7) && close_to(pooled[0], 7.463300277551, 1e-6));
}

void oracle_closed_forms()
{
    // uniform logits: ln V; one raised logit c among V - 1 zeros: ln(e^c + V - 1) - c e^c / (e^c + V - 1)
    const int V = 151936;
    std::vector<double> z((size_t)V, 0.0);
    double H;
    CHECK(oracle_entropy_from_logits(z.data(), 1, V, &H) == 0);
    CHECK(close_to(H, std::log((double)V), 1e-12));
    z[V - 1] = 5.0;
    CHECK(oracle_entropy_from_logits(z.data(), 1, V, &H) == 0);
    CHECK(std::fabs(H - 11.927305) < 1e-6);
    z[V - 1] = 0.0;
    z[0] = 12.0;
    CHECK(oracle_entropy_from_logits(z.data(), 1, V, &H) == 0);
    CHECK(std::fabs(H - 6.453048) < 1e-6);
    // one-hot hidden state picks a column of W (non-square, bf16 storage)
    const int d = 5, v = 7;
    std::vector<uint16_t> Wb((size_t)v * d), hb((size_t)d, 0);
    Rng r(3);
    for (auto &x : Wb)
        x = to_bf16((float)r.normal());
    hb[3] = to_bf16(1.0f);
    std::vector<double> logits((size_t)v);
    CHECK(oracle_logits(hb.data(), Wb.data(), 1, d, v, logits.data()) == 0);
    for (int i = 0; i < v; ++i) {
        uint32_t bits = (uint32_t)Wb[(size_t)i * d + 3] << 16;
        float f;
        std::memcpy(&f, &bits, 4);
        CHECK(logits[i] == (double)f);
    }
}

// every oracle entry point on ragged random data in exactly-sized heap buffers
void oracle_ragged_sweep()
{
    Rng r(11);
    for (int round = 0; round < 6; ++round) {
        const int B = 1 + r.below(7), d = 4 * (1 + r.below(5)), V = 3 + r.below(60), d_h = 1 + r.below(9);
        const int K = 1 + r.below(6), dtype = round & 1;
        std::vector<int32_t> len((size_t)B), off((size_t)B + 1);
        for (auto &l : len)
            l = r.below(4) == 0 ? 0 : r.below(9);
        CHECK(oracle_offsets(len.data(), B, off.data()) == 0);
        CHECK(off[0] == 0);
        const int64_t T = off[B];
        std::vector<int32_t> seg((size_t)T);
        CHECK(oracle_seg_ids(off.data(), B, T, seg.data()) == 0);
        for (int64_t t = 0; t < T; ++t)
            CHECK(off[seg[t]] <= t && t < off[seg[t] + 1]);
        const size_t es = dtype ? 2 : 4;
        std::vector<unsigned char> hid((size_t)T * d * es), W((size_t)V * d * es);
        auto fill = [&](std::vector<unsigned char> &buf, double scale) {
            for (size_t i = 0; i < buf.size() / es; ++i) {
                const float f = (float)(scale * r.normal());
                if (dtype) {
                    const uint16_t b = to_bf16(f);
                    std::memcpy(&buf[i * 2], &b, 2);
                } else {
                    std::memcpy(&buf[i * 4], &f, 4);
                }
            }
        };
        fill(hid, 1.0);
        fill(W, 1.0 / std::sqrt((double)d));
        std::vector<double> H((size_t)T), w((size_t)T), pooled((size_t)B * d), lse((size_t)B);
        CHECK(oracle_entropy(hid.data(), W.data(), dtype, T, d, V, H.data()) == 0);
        for (double h : H)
            CHECK(h >= -1e-12 && h <= std::log((double)V) + 1e-12);
        CHECK(oracle_pool(hid.data(), dtype, d, H.data(), off.data(), B, 1.0, w.data(), pooled.data(), lse.data()) == 0);
        for (int b = 0; b < B; ++b) {
            double sum = 0.0;
            for (int64_t t = off[b]; t < off[b + 1]; ++t)
                sum += w[(size_t)t];
            if (len[b] > 0)
                CHECK(close_to(sum, 1.0, 1e-12));
            else
                CHECK(std::isinf(lse[b]) && lse[b] < 0);
        }
        for (int kind = 0; kind < 3; ++kind) {
            std::vector<double> ab((size_t)B * d);
            CHECK(oracle_pool_ablation(hid.data(), dtype, d, off.data(), B, kind, ab.data()) == 0);
        }
        std::vector<float> w1((size_t)d_h * d), w2((size_t)K * d_h), b1((size_t)d_h), b2((size_t)K);
        for (auto &x : w1) x = (float)r.normal();
        for (auto &x : w2) x = (float)r.normal();
        for (auto &x : b1) x = (float)r.normal();
        for (auto &x : b2) x = (float)r.normal();
        std::vector<double> raw((size_t)B * K), p_hat((size_t)B * K), y_hat((size_t)B), centers((size_t)K);
        for (int k = 0; k < K; ++k)
            centers[(size_t)k] = 10.0 * (k + 1);
        CHECK(oracle_head(pooled.data(), B, d, d_h, K, w1.data(), b1.data(), w2.data(), b2.data(), 0, raw.data()) == 0);
        CHECK(oracle_head(pooled.data(), B, d, d_h, K, w1.data(), nullptr, w2.data(), nullptr, 0, raw.data()) == 0);
        CHECK(oracle_bin_decode(raw.data(), B, K, centers.data(), p_hat.data(), y_hat.data()) == 0);
        for (int b = 0; b < B; ++b) {
            double s = 0.0;
            for (int k = 0; k < K; ++k)
                s += p_hat[(size_t)b * K + k];
            CHECK(close_to(s, 1.0, 1e-12) && y_hat[b] >= 10.0 - 1e-9 && y_hat[b] <= 10.0 * K + 1e-9);
        }
        // training side
        std::vector<double> label((size_t)K);
        for (int i = 0; i < K; ++i) {
            CHECK(oracle_soft_label(i, K, label.data()) == 0);
            CHECK(close_to(std::accumulate(label.begin(), label.end(), 0.0), 1.0, 1e-12));
        }
        std::vector<double> x((size_t)B * d), yv((size_t)B), dw1(w1.begin(), w1.end()), db1(b1.begin(), b1.end()),
            dw2(w2.begin(), w2.end()), db2(b2.begin(), b2.end());
        std::vector<int32_t> bin((size_t)B);
        for (auto &v : x) v = r.normal();
        for (int b = 0; b < B; ++b) {
            bin[(size_t)b] = r.below(K);
            yv[(size_t)b] = centers[(size_t)bin[(size_t)b]] + r.normal();
        }
        std::vector<double> g1(dw1.size()), gb1(db1.size()), g2(dw2.size()), gb2(db2.size());
        double loss3[3];
        CHECK(oracle_head_loss_grad(x.data(), bin.data(), yv.data(), nullptr, B, d, d_h, K, dw1.data(), db1.data(),
                                    dw2.data(), db2.data(), centers.data(), 0.95, loss3, g1.data(), gb1.data(),
                                    g2.data(), gb2.data()) == 0);
        CHECK(std::isfinite(loss3[0]) && loss3[1] >= 0.0 && loss3[2] >= 0.0);
        CHECK(oracle_head_loss_grad(x.data(), bin.data(), yv.data(), nullptr, B, d, d_h, K, dw1.data(), db1.data(),
                                    dw2.data(), db2.data(), centers.data(), 0.95, loss3, nullptr, nullptr, nullptr,
                                    nullptr) == 0);
        std::vector<double> m(dw1.size(), 0.0), v(dw1.size(), 0.0), before(dw1);
        CHECK(oracle_adamw(dw1.data(), m.data(), v.data(), g1.data(), (int64_t)dw1.size(), 1e-3, 0.9, 0.999, 1e-8, 0.0,
                           1) == 0);
        for (size_t i = 0; i < dw1.size(); ++i)  // first step without decay: a move of lr against the gradient's sign
            if (std::fabs(g1[i]) > 1e-6)
                CHECK(close_to(before[i] - dw1[i], g1[i] > 0 ? 1e-3 : -1e-3, 1e-4));
    }
    // bad arguments are refused, not dereferenced
    CHECK(oracle_entropy(nullptr, nullptr, 0, 3, 2, 4, nullptr) != 0);
    CHECK(oracle_offsets(nullptr, 3, nullptr) != 0);
}

// ---- scheduling model -------------------------------------------------------------------------------------------
void sched_checks()
{
    // hand example: predictions order the jobs 2, 0, 3, 1; batches of 2 -> {2, 0}, {3, 1}
    const float pred[4] = {5.f, 9.f, 1.f, 7.f};
    const int32_t truth[4] = {6, 10, 2, 3};
    int32_t order[4];
    CHECK(egtp_sjf_order(pred, 4, order) == EGTP_OK);
    CHECK(order[0] == 2 && order[1] == 0 && order[2] == 3 && order[3] == 1);
    egtp_sched_report rep;
    int64_t done[4];
    int32_t batch_of[4];
    CHECK(egtp_simulate_batches(order, truth, 4, 2, &rep, done, batch_of) == EGTP_OK);
    CHECK(rep.n_batches == 2 && rep.actual_tokens == 21 && rep.allocated_tokens == 2 * 6 + 2 * 10);
    CHECK(rep.makespan_steps == 16 && done[2] == 2 && done[0] == 6 && done[3] == 9 && done[1] == 16);
    CHECK(close_to(rep.padding_ratio, 11.0 / 21.0, 1e-12));
    Rng r(5);
    for (int round = 0; round < 40; ++round) {
        const int n = r.below(70);
        const int bs = 1 + r.below(9);
        std::vector<float> p((size_t)n);
        std::vector<int32_t> tl((size_t)n), ord((size_t)n), bo((size_t)n);
        std::vector<int64_t> dn((size_t)n);
        for (int i = 0; i < n; ++i) {
            p[(size_t)i] = r.below(10) == 0 ? std::numeric_limits<float>::quiet_NaN() : (float)r.below(6);  // ties, NaNs
            tl[(size_t)i] = r.below(50);
        }
        CHECK(egtp_sjf_order(p.data(), n, ord.data()) == EGTP_OK);
        std::vector<char> seen((size_t)n, 0);
        for (int i = 0; i < n; ++i) {
            CHECK(ord[(size_t)i] >= 0 && ord[(size_t)i] < n && !seen[(size_t)ord[(size_t)i]]);
            seen[(size_t)ord[(size_t)i]] = 1;
            if (i > 0) {
                const float a = p[(size_t)ord[(size_t)i - 1]], b = p[(size_t)ord[(size_t)i]];
                CHECK(std::isnan(b) || a <= b);
                if (a == b || (std::isnan(a) && std::isnan(b)))
                    CHECK(ord[(size_t)i - 1] < ord[(size_t)i]);  // stable
            }
        }
        CHECK(egtp_simulate_batches(ord.data(), tl.data(), n, bs, &rep, dn.data(), bo.data()) == EGTP_OK);
        CHECK(rep.allocated_tokens >= rep.actual_tokens && rep.n_batches == (n + bs - 1) / bs);
        CHECK(egtp_simulate_batches(ord.data(), tl.data(), n, bs, &rep, nullptr, nullptr) == EGTP_OK);
        if (n > 1) {
            ord[0] = ord[1];  // no longer a permutation
            CHECK(egtp_simulate_batches(ord.data(), tl.data(), n, bs, &rep, nullptr, nullptr) == EGTP_ERR_OFFSETS);
        }
    }
    CHECK(egtp_sjf_order(nullptr, 3, order) == EGTP_ERR_NULL);
    CHECK(egtp_simulate_batches(order, truth, 4, 0, &rep, nullptr, nullptr) == EGTP_ERR_SHAPE);
}

// ---- launch plan: consistent for every size, and the workspace bounds really bound -------------------------------
void plan_checks()
{
    using namespace egtp;
    const int vocabs[] = {1, 255, 256, 257, 1000, 4096, 32000, 128037, 151936, 1 << 20};
    const int64_t big[] = {65536, 137720, 1000000, 16777216, 0x7fffffffLL};
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int V : vocabs) {
            size_t worst_part = 0, worst_pace = 0;
            auto one = [&](int64_t T) {
                const K1Plan p = k1_plan(dtype, T, 4096, V);
                CHECK(p.ntb == (T + p.tb_tokens - 1) / p.tb_tokens && p.ntiles_v == (V + p.tile_v - 1) / p.tile_v);
                CHECK(p.nsplit >= 1 && p.tiles_per_split >= 1);
                CHECK((int64_t)p.nsplit * p.tiles_per_split >= p.ntiles_v);           // the ranges cover the vocabulary
                CHECK((int64_t)(p.nsplit - 1) * p.tiles_per_split < p.ntiles_v);      // and none of them is empty
                const size_t part = k1_partial_floats(p, T);
                const size_t pace = (size_t)8 * (size_t)k1_pace_cohorts((long)p.ntb * p.nsplit);
                worst_part = part > worst_part ? part : worst_part;
                worst_pace = pace > worst_pace ? pace : worst_pace;
                // a workspace sized for T serves every smaller batch: the bounds cover the worst seen so far
                CHECK(k1_partial_floats_bound(T) >= worst_part);
                CHECK(k1_pace_ints_bound(T) >= worst_pace);
            };
            for (int64_t T = 1; T <= 6000; ++T)
                one(T);
            for (int64_t T : big)
                for (int64_t dT = -2; dT <= 0; ++dT)
                    one(T + dT);
        }
    // the paced configuration is the one with more than K1_PACE_TILES tiles per range
    const K1Plan serving = k1_plan(DT_BF16, 137720, 4096, 151936);
    CHECK(serving.tiles_per_split > K1_PACE_TILES && k1_plan_paces(serving));
    // fp32 operands run the same kernel over a contraction six times as long, in whole 32-element segments
    CHECK(k1_contraction_len(DT_BF16, 4096) == 4096 && k1_contraction_len(DT_F32, 4096) == 6 * 4096);
    CHECK(k1_contraction_len(DT_F32, 4) == 6 * 32 && k1_contraction_len(DT_F32, 36) == 6 * 64);
    CHECK(k1_contraction_len(DT_F32, 699040) <= K1_MAX_CONTRACTION && k1_contraction_len(DT_F32, 699044) > K1_MAX_CONTRACTION);
    const K1Plan serving_f32 = k1_plan(DT_F32, 137720, 4096, 151936);
    CHECK(serving_f32.nsplit == serving.nsplit && serving_f32.tb_tokens == serving.tb_tokens);
    // 512 decode tokens: two token blocks, and one round of workgroups rather than five rounds of single tiles
    const K1Plan decode = k1_plan(DT_BF16, 512, 4096, 151936);
    CHECK(decode.ntb == 2 && (long)decode.ntb * decode.nsplit <= 256 && decode.tiles_per_split == 5);
    const K1Plan one_tile = k1_plan(DT_BF16, 10, 64, 200);
    CHECK(one_tile.nsplit == 1 && one_tile.tiles_per_split == 1 && !k1_plan_paces(one_tile));
}

}  // namespace

int main()
{
    oracle_worked_example();
    oracle_closed_forms();
    oracle_ragged_sweep();
    sched_checks();
    plan_checks();
    if (failures) {
        std::fprintf(stderr, "%d check(s) failed\n", failures);
        return 1;
    }
    std::puts("host checks passed under the sanitizers");
    return 0;
}
