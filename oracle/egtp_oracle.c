/*
 * egtp_oracle.c -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, fp64 CPU statement of what Entropy-Guided Token Pooling (EGTP)
 * and Progressive Length Prediction (PLP) compute, written from the paper's
 * equations so that a reader can check each function against the paper by eye.
 * Only the test-suite, the smoke check and the benchmark's CPU-baseline leg may
 * call it.  It shares nothing with the GPU library: no headers, no helpers, no
 * tables.  There is no tiling, no streaming, no fusion and no reordering of any
 * sum: every reduction is the definition written out (two passes where the
 * definition needs a maximum or a normaliser first).
 *
 * Inputs arrive with the bit patterns the GPU receives (fp32, or bf16 stored as
 * the upper 16 bits of an fp32) and are widened exactly to fp64; nothing is ever
 * rounded back to a narrower type.  The only parallelism is an OpenMP
 * "parallel for" over independent tokens / sequences.
 *
 * Pins (tests under tests/, CPU only): closed forms for the entropy (uniform,
 * one-hot-ish, k-level logits, dyadic distribution), shift / permutation /
 * vocabulary-duplication invariants, library cross-checks (scipy softmax+entr,
 * logsumexp), mean-pooling and single-token special cases, the merge law,
 * brute force in exact rational arithmetic, and a hand-derived worked example.
 * The training objective of the head (Eq. 5-7, Eq. 9 as per-sample weights, AdamW)
 * is pinned by closed forms of the soft label, central finite differences of the
 * loss for every gradient, torch's autograd and torch.optim.AdamW in fp64 on the
 * CPU, and the closed form of the first AdamW step.
 * Parity unpinned (stated here and in the design notes): the meaning of a
 * temperature alpha != 1 (Eq. 3 prints no alpha; this file divides H by alpha),
 * and any bin centres for the K-bin decode (the paper never gives them; the
 * caller supplies them).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_F32 = 0, ORC_BF16 = 1, ORC_F64 = 2 };

enum { ORC_OK = 0, ORC_BAD_ARG = 1, ORC_NO_MEM = 2 };

/* exact widening of element idx of an array of the given storage type */
static double widen(const void *p, int dtype, int64_t idx)
{
    if (dtype == ORC_F32)
        return (double)((const float *)p)[idx];
    if (dtype == ORC_BF16) {
        uint32_t bits = (uint32_t)((const uint16_t *)p)[idx] << 16;
        float f;
        memcpy(&f, &bits, sizeof f);
        return (double)f;
    }
    return ((const double *)p)[idx];
}

/* ------------------------------------------------------------------------- */
/* Ragged plumbing: offsets are the running sum of the lengths; the segment of */
/* a token is found by walking the offsets.                                    */
/* ------------------------------------------------------------------------- */

int oracle_offsets(const int32_t *lengths, int32_t B, int32_t *offsets)
{
    if (B < 0 || !offsets || (B > 0 && !lengths))
        return ORC_BAD_ARG;
    int64_t run = 0;
    offsets[0] = 0;
    for (int32_t b = 0; b < B; ++b) {
        if (lengths[b] < 0)
            return ORC_BAD_ARG;
        run += lengths[b];
        if (run > INT32_MAX)
            return ORC_BAD_ARG;
        offsets[b + 1] = (int32_t)run;
    }
    return ORC_OK;
}

int oracle_seg_ids(const int32_t *offsets, int32_t B, int64_t T, int32_t *seg)
{
    if (B < 0 || T < 0 || !offsets || (T > 0 && !seg))
        return ORC_BAD_ARG;
    for (int64_t t = 0; t < T; ++t) {
        int32_t found = -1;
        for (int32_t b = 0; b < B; ++b)
            if (offsets[b] <= t && t < offsets[b + 1]) {
                found = b;
                break;
            }
        seg[t] = found;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Eq. 2: entropy of the next-token distribution, H = -sum_v P(v) log P(v),    */
/* natural log, with P = softmax of the logits.                               */
/* ------------------------------------------------------------------------- */

/* entropy (nats) of softmax(z[0..V)) -- the definition, via log-probabilities */
static double softmax_entropy(const double *z, int32_t V)
{
    double m = -INFINITY;
    for (int32_t v = 0; v < V; ++v)
        if (z[v] > m)
            m = z[v];
    double S = 0.0;
    for (int32_t v = 0; v < V; ++v)
        S += exp(z[v] - m);
    double lnS = log(S);
    double H = 0.0;
    for (int32_t v = 0; v < V; ++v) {
        double lnp = (z[v] - m) - lnS;
        double p = exp(lnp);
        if (p > 0.0) /* lim p->0 of p ln p is 0 */
            H -= p * lnp;
    }
    return H;
}

/* H[t] for T rows of V given logits (fp64, row-major) */
int oracle_entropy_from_logits(const double *z, int64_t T, int32_t V, double *H)
{
    if (T < 0 || V <= 0 || (T > 0 && (!z || !H)))
        return ORC_BAD_ARG;
    for (int64_t t = 0; t < T; ++t)
        H[t] = softmax_entropy(z + t * (int64_t)V, V);
    return ORC_OK;
}

/* logits of one token: z[v] = sum_k W_lm[v,k] * h[k]; W_lm is [V x d] row-major */
int oracle_logits(const void *hidden_row, const void *w_lm, int dtype, int32_t d, int32_t V,
                  double *z)
{
    if (d <= 0 || V <= 0 || !hidden_row || !w_lm || !z)
        return ORC_BAD_ARG;
    for (int32_t v = 0; v < V; ++v) {
        double acc = 0.0;
        for (int32_t k = 0; k < d; ++k)
            acc += widen(w_lm, dtype, (int64_t)v * d + k) * widen(hidden_row, dtype, k);
        z[v] = acc;
    }
    return ORC_OK;
}

/* Eq. 2 for every token of hidden[T x d] against the LM head w_lm[V x d] */
int oracle_entropy(const void *hidden, const void *w_lm, int dtype, int64_t T, int32_t d,
                   int32_t V, double *H)
{
    if (T < 0 || d <= 0 || V <= 0 || !w_lm || (T > 0 && (!hidden || !H)))
        return ORC_BAD_ARG;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t t = 0; t < T; ++t) {
        double *h = (double *)malloc(sizeof(double) * (size_t)d);
        double *z = (double *)malloc(sizeof(double) * (size_t)V);
        if (!h || !z) {
            failed = 1;
        } else {
            for (int32_t k = 0; k < d; ++k)
                h[k] = widen(hidden, dtype, t * (int64_t)d + k);
            for (int32_t v = 0; v < V; ++v) {
                double acc = 0.0;
                for (int32_t k = 0; k < d; ++k)
                    acc += widen(w_lm, dtype, (int64_t)v * d + k) * h[k];
                z[v] = acc;
            }
            H[t] = softmax_entropy(z, V);
        }
        free(h);
        free(z);
    }
    return failed ? ORC_NO_MEM : ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Eq. 3 and Eq. 4: w_i = exp(H_i/alpha) / sum_j exp(H_j/alpha) inside each    */
/* sequence (alpha = 1 is the equation as printed), pooled = sum_i w_i h_i.    */
/* lse = log sum_j exp(H_j/alpha).  An empty sequence gives pooled = 0 and     */
/* lse = -inf.  w (length T) may be NULL.                                      */
/* ------------------------------------------------------------------------- */

int oracle_pool(const void *hidden, int dtype, int32_t d, const double *H, const int32_t *offsets,
                int32_t B, double alpha, double *w, double *pooled, double *lse)
{
    if (d <= 0 || B < 0 || !(alpha > 0.0) || !offsets || (B > 0 && (!pooled || !lse)))
        return ORC_BAD_ARG;
    if (offsets[0] != 0)
        return ORC_BAD_ARG;
    for (int32_t b = 0; b < B; ++b)
        if (offsets[b + 1] < offsets[b])
            return ORC_BAD_ARG;
    if (offsets[B] > 0 && (!hidden || !H))
        return ORC_BAD_ARG;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        int64_t lo = offsets[b], hi = offsets[b + 1];
        double *out = pooled + (int64_t)b * d;
        for (int32_t k = 0; k < d; ++k)
            out[k] = 0.0;
        if (hi == lo) {
            lse[b] = -INFINITY;
            continue;
        }
        double M = -INFINITY;
        for (int64_t i = lo; i < hi; ++i)
            if (H[i] / alpha > M)
                M = H[i] / alpha;
        double D = 0.0;
        for (int64_t i = lo; i < hi; ++i)
            D += exp(H[i] / alpha - M);
        lse[b] = M + log(D);
        for (int64_t i = lo; i < hi; ++i) {
            double wi = exp(H[i] / alpha - M) / D;
            if (w)
                w[i] = wi;
            for (int32_t k = 0; k < d; ++k)
                out[k] += wi * widen(hidden, dtype, i * (int64_t)d + k);
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* The pooling alternatives of the ablation (Table 3): average, max, last.     */
/* kind: 0 = average, 1 = element-wise max, 2 = last token.  Empty sequence    */
/* gives the zero vector.                                                      */
/* ------------------------------------------------------------------------- */

int oracle_pool_ablation(const void *hidden, int dtype, int32_t d, const int32_t *offsets,
                         int32_t B, int kind, double *pooled)
{
    if (d <= 0 || B < 0 || !offsets || kind < 0 || kind > 2 || (B > 0 && !pooled))
        return ORC_BAD_ARG;
    for (int32_t b = 0; b < B; ++b) {
        int64_t lo = offsets[b], hi = offsets[b + 1];
        double *out = pooled + (int64_t)b * d;
        for (int32_t k = 0; k < d; ++k) {
            if (hi <= lo) {
                out[k] = 0.0;
            } else if (kind == 0) {
                double s = 0.0;
                for (int64_t i = lo; i < hi; ++i)
                    s += widen(hidden, dtype, i * (int64_t)d + k);
                out[k] = s / (double)(hi - lo);
            } else if (kind == 1) {
                double mx = -INFINITY;
                for (int64_t i = lo; i < hi; ++i) {
                    double x = widen(hidden, dtype, i * (int64_t)d + k);
                    if (x > mx)
                        mx = x;
                }
                out[k] = mx;
            } else {
                out[k] = widen(hidden, dtype, (hi - 1) * (int64_t)d + k);
            }
        }
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Prediction head (Section 3.2): a two-layer perceptron on the pooled vector. */
/* out[b, o] = b2[o] + sum_j w2[o, j] * max(0, b1[j] + sum_k w1[j, k] x[b, k]). */
/* w1 is [d_h x d], w2 is [n_out x d_h], row-major, storage type wdtype;        */
/* biases are fp32 and may be NULL (= 0).                                      */
/* ------------------------------------------------------------------------- */

int oracle_head(const double *x, int32_t B, int32_t d, int32_t d_h, int32_t n_out, const void *w1,
                const float *b1, const void *w2, const float *b2, int wdtype, double *out)
{
    if (B < 0 || d <= 0 || d_h <= 0 || n_out <= 0 || !w1 || !w2 || (B > 0 && (!x || !out)))
        return ORC_BAD_ARG;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t b = 0; b < B; ++b) {
        double *a = (double *)malloc(sizeof(double) * (size_t)d_h);
        if (!a) {
            failed = 1;
            continue;
        }
        for (int32_t j = 0; j < d_h; ++j) {
            double pre = b1 ? (double)b1[j] : 0.0;
            for (int32_t k = 0; k < d; ++k)
                pre += widen(w1, wdtype, (int64_t)j * d + k) * x[(int64_t)b * d + k];
            a[j] = pre > 0.0 ? pre : 0.0;
        }
        for (int32_t o = 0; o < n_out; ++o) {
            double y = b2 ? (double)b2[o] : 0.0;
            for (int32_t j = 0; j < d_h; ++j)
                y += widen(w2, wdtype, (int64_t)o * d_h + j) * a[j];
            out[(int64_t)b * n_out + o] = y;
        }
        free(a);
    }
    return failed ? ORC_NO_MEM : ORC_OK;
}

/* Eq. 6: p_hat = softmax over the K head outputs, y_hat = sum_i p_hat_i c_i */
int oracle_bin_decode(const double *logits, int32_t B, int32_t K, const double *centers,
                      double *p_hat, double *y_hat)
{
    if (B < 0 || K <= 0 || !centers || (B > 0 && (!logits || !y_hat)))
        return ORC_BAD_ARG;
    for (int32_t b = 0; b < B; ++b) {
        const double *z = logits + (int64_t)b * K;
        double m = -INFINITY;
        for (int32_t i = 0; i < K; ++i)
            if (z[i] > m)
                m = z[i];
        double S = 0.0;
        for (int32_t i = 0; i < K; ++i)
            S += exp(z[i] - m);
        double y = 0.0;
        for (int32_t i = 0; i < K; ++i) {
            double p = exp(z[i] - m) / S;
            if (p_hat)
                p_hat[(int64_t)b * K + i] = p;
            y += p * centers[i];
        }
        y_hat[b] = y;
    }
    return ORC_OK;
}

/* ------------------------------------------------------------------------- */
/* Training objective of the prediction head on frozen pooled features         */
/* (Section 3.2, Eq. 5-7; Eq. 9 through per-sample weights).                   */
/* ------------------------------------------------------------------------- */

/* Eq. 5: soft label over K bins for a target that falls into bin i (0-based):  */
/* p_j = exp(-|j - i|) / sum_k exp(-|k - i|).                                   */
int oracle_soft_label(int32_t i, int32_t K, double *p)
{
    if (K <= 0 || i < 0 || i >= K || !p)
        return ORC_BAD_ARG;
    double Z = 0.0;
    for (int32_t k = 0; k < K; ++k)
        Z += exp(-fabs((double)(k - i)));
    for (int32_t j = 0; j < K; ++j)
        p[j] = exp(-fabs((double)(j - i))) / Z;
    return ORC_OK;
}

/* Eq. 7 with its gradient.  Parameters are fp64 here: w1[d_h x d], b1[d_h], w2[K x d_h],    */
/* b2[K]; x[B x d] pooled features; bin[B] the target's bin, y[B] the target length;          */
/* weight[B] per-sample weights (NULL = 1/B each; Eq. 9 averages a sequence's steps by        */
/* giving each of its T steps weight 1/(N T)); c[K] bin centres.                              */
/*   loss = sum_b weight_b ( lambda * CE_b + (1 - lambda) * (y_b - yhat_b)^2 ),               */
/*   CE_b = - sum_j p_bj log phat_bj,  phat_b = softmax(z_b),  yhat_b = sum_j phat_bj c_j,     */
/*   z_b = w2 relu(w1 x_b + b1) + b2.                                                         */
/* loss3 = {total, weighted CE part, weighted MSE part} (each before the lambda factors for   */
/* the two parts).  Gradients may each be NULL.                                               */
int oracle_head_loss_grad(const double *x, const int32_t *bin, const double *y, const double *weight,
                          int32_t B, int32_t d, int32_t d_h, int32_t K, const double *w1,
                          const double *b1, const double *w2, const double *b2, const double *c,
                          double lambda, double *loss3, double *g_w1, double *g_b1, double *g_w2,
                          double *g_b2)
{
    if (B <= 0 || d <= 0 || d_h <= 0 || K <= 0 || !x || !bin || !y || !w1 || !b1 || !w2 || !b2 || !c || !loss3)
        return ORC_BAD_ARG;
    if (g_w1) memset(g_w1, 0, sizeof(double) * (size_t)d_h * d);
    if (g_b1) memset(g_b1, 0, sizeof(double) * (size_t)d_h);
    if (g_w2) memset(g_w2, 0, sizeof(double) * (size_t)K * d_h);
    if (g_b2) memset(g_b2, 0, sizeof(double) * (size_t)K);
    double *a = (double *)malloc(sizeof(double) * (size_t)d_h);
    double *da = (double *)malloc(sizeof(double) * (size_t)d_h);
    double *z = (double *)malloc(sizeof(double) * (size_t)K);
    double *ph = (double *)malloc(sizeof(double) * (size_t)K);
    double *p = (double *)malloc(sizeof(double) * (size_t)K);
    double *dz = (double *)malloc(sizeof(double) * (size_t)K);
    if (!a || !da || !z || !ph || !p || !dz) {
        free(a); free(da); free(z); free(ph); free(p); free(dz);
        return ORC_NO_MEM;
    }
    double ce_sum = 0.0, mse_sum = 0.0;
    int rc = ORC_OK;
    for (int32_t b = 0; b < B && rc == ORC_OK; ++b) {
        const double wb = weight ? weight[b] : 1.0 / (double)B;
        const double *xb = x + (int64_t)b * d;
        for (int32_t j = 0; j < d_h; ++j) {
            double pre = b1[j];
            for (int32_t k = 0; k < d; ++k)
                pre += w1[(int64_t)j * d + k] * xb[k];
            a[j] = pre > 0.0 ? pre : 0.0;
        }
        double m = -INFINITY;
        for (int32_t o = 0; o < K; ++o) {
            double s = b2[o];
            for (int32_t j = 0; j < d_h; ++j)
                s += w2[(int64_t)o * d_h + j] * a[j];
            z[o] = s;
            if (s > m) m = s;
        }
        double S = 0.0;
        for (int32_t o = 0; o < K; ++o)
            S += exp(z[o] - m);
        double yhat = 0.0;
        for (int32_t o = 0; o < K; ++o) {
            ph[o] = exp(z[o] - m) / S;
            yhat += ph[o] * c[o];
        }
        rc = oracle_soft_label(bin[b], K, p);
        if (rc != ORC_OK)
            break;
        double ce = 0.0;
        for (int32_t o = 0; o < K; ++o)
            ce -= p[o] * ((z[o] - m) - log(S));
        const double err = yhat - y[b];
        ce_sum += wb * ce;
        mse_sum += wb * err * err;
        /* d loss / d z_o = wb ( lambda (phat_o - p_o) + (1-lambda) 2 err phat_o (c_o - yhat) ) */
        for (int32_t o = 0; o < K; ++o)
            dz[o] = wb * (lambda * (ph[o] - p[o]) + (1.0 - lambda) * 2.0 * err * ph[o] * (c[o] - yhat));
        for (int32_t j = 0; j < d_h; ++j) {
            double s = 0.0;
            for (int32_t o = 0; o < K; ++o)
                s += dz[o] * w2[(int64_t)o * d_h + j];
            da[j] = a[j] > 0.0 ? s : 0.0;
        }
        for (int32_t o = 0; o < K; ++o) {
            if (g_b2) g_b2[o] += dz[o];
            if (g_w2)
                for (int32_t j = 0; j < d_h; ++j)
                    g_w2[(int64_t)o * d_h + j] += dz[o] * a[j];
        }
        for (int32_t j = 0; j < d_h; ++j) {
            if (g_b1) g_b1[j] += da[j];
            if (g_w1 && da[j] != 0.0)
                for (int32_t k = 0; k < d; ++k)
                    g_w1[(int64_t)j * d + k] += da[j] * xb[k];
        }
    }
    loss3[0] = lambda * ce_sum + (1.0 - lambda) * mse_sum;
    loss3[1] = ce_sum;
    loss3[2] = mse_sum;
    free(a); free(da); free(z); free(ph); free(p); free(dz);
    return rc;
}

/* AdamW (decoupled weight decay), one step t >= 1 on n parameters:                         */
/*   m = b1 m + (1-b1) g;  v = b2 v + (1-b2) g^2;  mhat = m/(1-b1^t);  vhat = v/(1-b2^t);    */
/*   w = w - lr * wd * w - lr * mhat / (sqrt(vhat) + eps).                                   */
int oracle_adamw(double *w, double *m, double *v, const double *g, int64_t n, double lr, double beta1,
                 double beta2, double eps, double weight_decay, int64_t t)
{
    if (n < 0 || t < 1 || (n > 0 && (!w || !m || !v || !g)))
        return ORC_BAD_ARG;
    const double c1 = 1.0 - pow(beta1, (double)t), c2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        m[i] = beta1 * m[i] + (1.0 - beta1) * g[i];
        v[i] = beta2 * v[i] + (1.0 - beta2) * g[i] * g[i];
        const double mhat = m[i] / c1, vhat = v[i] / c2;
        w[i] = w[i] - lr * weight_decay * w[i] - lr * mhat / (sqrt(vhat) + eps);
    }
    return ORC_OK;
}
