/*
 * egtp.h -- C ABI of the MI355X (gfx950) library for Entropy-Guided Token Pooling (EGTP)
 * and Progressive Length Prediction (PLP) scoring.
 *
 * What the calls compute (paper, Section 3):
 *   Eq. 2   per-token entropy H_i (nats) of softmax(W_lm h_i) over the full vocabulary;
 *   Eq. 3   per-sequence weights  w_i = exp(H_i/alpha) / sum_j exp(H_j/alpha)  (alpha = 1 is
 *           the equation as printed; the text mentions a temperature without placing it);
 *   Eq. 4   pooled vector  h = sum_i w_i h_i ;
 *   Sec 3.2 prediction head on h: a perceptron d -> d_h (ReLU) -> n_out.  n_out == 1 gives the
 *           length directly; n_out == K > 1 applies Eq. 6 (softmax over K bins, expected value
 *           over the caller's bin centres);
 *   Eq. 8   PLP: the same head (or a second one) on a representation that aggregates the prompt
 *           with every token generated so far.  Aggregation here is the running entropy-weighted
 *           pool, carried as the pair (pooled, lse): folding tokens into that pair gives exactly
 *           the EGTP pooling of the prompt followed by the generated tokens.
 *
 * Conventions
 *   - Pointers named *_dev / hidden / w_lm / head weights / outputs / workspace / state are HIP
 *     device pointers on the device that was current at egtp_create; *_host are host pointers.
 *   - Every pointer is borrowed.  egtp_score / plp_step / egtp_build_offsets allocate nothing:
 *     the caller brings a workspace of egtp_workspace_bytes().  They only enqueue work on the
 *     given stream (a hipStream_t passed as void*, NULL = default stream) and return; outputs are
 *     valid once the stream has been synchronised.  The workspace must not be shared by calls
 *     that may overlap in time.
 *   - Matrices are row-major, dense.  hidden is [T x d], w_lm is [vocab x d], both of
 *     egtp_config.dtype (bf16 = upper half of an fp32, or fp32).  Accumulation, entropies,
 *     pooled vectors, lse and predictions are fp32.  Row starts must be 16-byte aligned
 *     (bf16: d a multiple of 8; fp32: d a multiple of 4).  The LM-head contraction of Eq. 2 runs
 *     on the bf16 matrix cores for both types: products of bf16 values are exact in the fp32
 *     accumulators; an fp32 value enters as the exact sum of three bf16 pieces, and of the nine
 *     piece products of w*h the six of relative size >= 2^-16 are accumulated (the rest is below
 *     fp32's own rounding), so fp32 inputs give fp32-grade logits at six times the bf16 cost.
 *   - Ragged batches: offsets[B+1] int32, offsets[0] = 0, non-decreasing, offsets[B] = T.
 *     A repeated offset is an empty sequence: pooled = 0, lse = -inf, prediction = head(0).
 *   - Errors are return codes; on any error nothing has been launched.  B == 0 or T == 0 with
 *     B == 0 is EGTP_OK and launches nothing.  NaN/Inf inputs are not screened.
 *   - Results are deterministic: no floating-point atomics, fixed reduction orders.
 *   - A context is not thread-safe; distinct contexts are independent.
 */
#ifndef EGTP_H
#define EGTP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct egtp_ctx egtp_ctx; /* opaque */

typedef enum {
    EGTP_OK = 0,
    EGTP_ERR_NULL = 1,      /* a required pointer is NULL */
    EGTP_ERR_SHAPE = 2,     /* a size is negative, zero where it may not be, or unsupported */
    EGTP_ERR_OFFSETS = 3,   /* host offsets mirror is malformed */
    EGTP_ERR_DTYPE = 4,     /* unknown storage type */
    EGTP_ERR_WORKSPACE = 5, /* workspace NULL, misaligned (256 B) or too small */
    EGTP_ERR_ARCH = 6,      /* current device is not gfx950 */
    EGTP_ERR_HIP = 7,       /* a HIP call failed; see egtp_last_hip_error */
    EGTP_ERR_ALPHA = 8,     /* temperature not a finite number > 0 */
    EGTP_ERR_HYPER = 9      /* a training hyper-parameter is outside its range */
} egtp_status;

typedef enum { EGTP_F32 = 0, EGTP_BF16 = 1 } egtp_dtype;

/* Pooling alternatives of the paper's ablation (Table 3). */
typedef enum { EGTP_POOL_AVERAGE = 0, EGTP_POOL_MAX = 1, EGTP_POOL_LAST = 2 } egtp_pool_kind;

/* One prediction head (Section 3.2): x[d] -> relu(w1 x + b1)[d_h] -> w2 . + b2 [n_out]. */
typedef struct {
    int32_t d_h;              /* hidden width, 1 .. 16384 */
    int32_t n_out;            /* 1 = scalar length; K > 1 = K-bin head decoded with Eq. 6 (K <= 1024) */
    egtp_dtype wdtype;        /* storage type of w1 and w2 */
    const void *w1;           /* [d_h x d]     device */
    const float *b1;          /* [d_h]         device, NULL = zeros */
    const void *w2;           /* [n_out x d_h] device */
    const float *b2;          /* [n_out]       device, NULL = zeros */
    const float *bin_centers; /* [n_out]       device; required iff n_out > 1 (the c_i of Eq. 6) */
} egtp_head;

typedef struct {
    int32_t d;          /* hidden size (bf16: at most 4 194 240; fp32: at most 699 040) */
    int32_t vocab;      /* vocabulary size V */
    egtp_dtype dtype;   /* storage type of hidden states and w_lm */
    const void *w_lm;   /* [vocab x d] device, must outlive the context.  May be NULL: the context then
                         * lives on a packed copy alone (egtp_adopt_packed_w_lm) */
    float alpha;        /* pooling temperature, finite and > 0; 1.0f is Eq. 3 as printed */
    egtp_head head_len; /* EGTP: predicted total length */
    egtp_head head_rem; /* PLP: predicted remaining length; w1 == NULL means "use head_len" */
} egtp_config;

/* Validates the configuration, checks that the current device is gfx950 and records it.
 * Makes no large allocation.  *out is set only on EGTP_OK. */
egtp_status egtp_create(const egtp_config *cfg, egtp_ctx **out);
egtp_status egtp_destroy(egtp_ctx *ctx);

/* The matrix-core kernel reads W_lm from a packed copy (tiles of 256 rows x 32 K elements of bf16,
 * contiguous per tile and K step; 2 bytes per element of W_lm for bf16, 12 for fp32: six K segments
 * of bf16 pieces).  egtp_pack_w_lm builds that copy once into
 * packed_dev (device memory of at least egtp_packed_w_lm_bytes(), 256-byte aligned, borrowed:
 * it must stay valid and unmodified while the context uses it; enqueued on `stream`, and later
 * scoring calls must be ordered after it).  Without it every scoring call re-packs W_lm into
 * its workspace first -- fine for large prefill batches, wasteful for decode steps.  Calling it
 * again re-packs (after w_lm changed); packed_dev == NULL forgets the copy.  Changing between
 * "packed" and "not packed" changes egtp_workspace_bytes().  A context created with
 * w_lm == NULL has nothing to pack from (EGTP_ERR_NULL). */
size_t egtp_packed_w_lm_bytes(const egtp_ctx *ctx);
egtp_status egtp_pack_w_lm(egtp_ctx *ctx, void *packed_dev, size_t bytes, void *stream);
/* Registers a packed copy that already exists -- built earlier by egtp_pack_w_lm of a context with
 * the same d, vocab and dtype -- without touching it.  With it a context needs no row-major W_lm at
 * all: the Eq. 2 kernel only ever reads the packed copy, so a caller that keeps W_lm elsewhere (or
 * nowhere) saves the d vocab elements of the row-major matrix.  Same alignment, size and lifetime rules as above; scoring
 * calls of a context that has neither w_lm nor a packed copy return EGTP_ERR_NULL. */
egtp_status egtp_adopt_packed_w_lm(egtp_ctx *ctx, const void *packed_dev, size_t bytes);

/* Bytes of workspace sufficient for any egtp_score / plp_step / egtp_pool_ablation call with
 * at most max_tokens tokens and max_seqs sequences.  0 if an argument is invalid. */
size_t egtp_workspace_bytes(const egtp_ctx *ctx, int64_t max_tokens, int32_t max_seqs);

const char *egtp_status_string(egtp_status s);
/* The hipError_t (as int) of the last failed HIP call made through this context, 0 if none. */
int egtp_last_hip_error(const egtp_ctx *ctx);

/* Ragged plumbing: offsets_dev[B+1] = exclusive prefix sum of lengths_dev[B] (int32; the caller
 * guarantees the total fits), and, if seg_ids_dev != NULL, seg_ids_dev[t] = the sequence b with
 * offsets[b] <= t < offsets[b+1] for t < T.  Integer work, exact. */
egtp_status egtp_build_offsets(egtp_ctx *ctx, const int32_t *lengths_dev, int32_t B,
                               int32_t *offsets_dev, int32_t *seg_ids_dev, int64_t T, void *stream);

/* EGTP over one ragged batch (Eq. 2 -> Eq. 3 -> Eq. 4 -> head_len).
 *   hidden        [T x d] cfg.dtype
 *   offsets_dev   [B+1] device
 *   offsets_host  optional host copy of the same offsets; when given it is checked here
 *                 (EGTP_ERR_OFFSETS) before anything is launched
 *   entropy_out   [T] fp32, optional (NULL: kept in the workspace only)
 *   pooled_out    [B x d] fp32   \  together the PLP state of each sequence
 *   lse_out       [B] fp32       /  lse_b = log sum_i exp(H_i/alpha)
 *   pred_out      [B] fp32, predicted length
 * No [T x vocab] logits tensor is written anywhere. */
egtp_status egtp_score(egtp_ctx *ctx, const void *hidden, const int32_t *offsets_dev,
                       const int32_t *offsets_host, int32_t B, int64_t T, void *workspace,
                       size_t workspace_bytes, float *entropy_out, float *pooled_out,
                       float *lse_out, float *pred_out, void *stream);

/* egtp_score for a K-bin head (head_len.n_out = K > 1) that also hands out the distribution the
 * predicted length is the expectation of (Eq. 6): p_hat_out [B x K] fp32, row b = softmax over the
 * K head outputs of sequence b (each row sums to 1; pred_out[b] = sum_j p_hat[b][j] c_j).
 * A scalar head (n_out == 1) is EGTP_ERR_SHAPE; everything else as egtp_score. */
egtp_status egtp_score_dist(egtp_ctx *ctx, const void *hidden, const int32_t *offsets_dev,
                            const int32_t *offsets_host, int32_t B, int64_t T, void *workspace,
                            size_t workspace_bytes, float *entropy_out, float *pooled_out,
                            float *lse_out, float *pred_out, float *p_hat_out, void *stream);

/* One PLP update (Eq. 8) for B live sequences: fold new tokens into each sequence's running
 * state and predict the remaining length with head_rem.
 *   hidden_new       [T_new x d] hidden states of the newly generated tokens
 *   offsets_new_dev  [B+1] ragged offsets of the new tokens, or NULL = exactly one new token per
 *                    sequence (then T_new must equal B)
 *   offsets_new_host optional host mirror, checked like egtp_score's
 *   slot_dev         optional [B]: sequence b lives in state row slot[b] (distinct, >= 0);
 *                    NULL = row b
 *   pooled_state     [S x d] fp32 in/out,  lse_state [S] fp32 in/out.  The empty state is
 *                    (zeros, -inf); egtp_score's (pooled_out, lse_out) is the state after the prompt
 *   entropy_out      [T_new] optional
 *   rem_pred_out     [B] predicted remaining length
 * With state (p, L) and new tokens (h_i, H_i):  L' = log(e^L + sum_i e^{H_i/alpha}),
 * p' = p e^{L-L'} + sum_i h_i e^{H_i/alpha - L'}. */
egtp_status plp_step(egtp_ctx *ctx, const void *hidden_new, const int32_t *offsets_new_dev,
                     const int32_t *offsets_new_host, const int32_t *slot_dev, int32_t B,
                     int64_t T_new, float *pooled_state, float *lse_state, void *workspace,
                     size_t workspace_bytes, float *entropy_out, float *rem_pred_out, void *stream);

/* plp_step for a K-bin remaining-length head, also writing its distribution (Eq. 6):
 * p_hat_out [B x K] fp32 as in egtp_score_dist (row b belongs to sequence b, whatever its slot). */
egtp_status plp_step_dist(egtp_ctx *ctx, const void *hidden_new, const int32_t *offsets_new_dev,
                          const int32_t *offsets_new_host, const int32_t *slot_dev, int32_t B,
                          int64_t T_new, float *pooled_state, float *lse_state, void *workspace,
                          size_t workspace_bytes, float *entropy_out, float *rem_pred_out,
                          float *p_hat_out, void *stream);

/* plp_step for callers that cannot allocate device memory and have no workspace to bring: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The same kernels
 * as plp_step, run on a scratch array that is part of the library itself: EGTP_STATIC_SCRATCH_BYTES
 * of device memory, present on every device the library is loaded on until the process ends.  The
 * call allocates and frees nothing.
 *   - Limit: egtp_workspace_bytes(ctx, T_new, B) must not exceed egtp_static_scratch_bytes()
 *     (64 MiB: enough for 512 sequences x 1 token at d = 5120, vocab = 151936, d_h = 1280 with a
 *     packed W_lm registered -- without one the per-call packed copy alone is over the limit);
 *     otherwise EGTP_ERR_WORKSPACE and nothing is launched.  Larger batches are the caller's to split.
 *   - The current device must be the context's (EGTP_ERR_ARCH otherwise).
 *   - Every call on a device uses that device's one array, whatever the context or stream: calls
 *     that may overlap in time on one device race.  Order them on one stream or with events.  The
 *     array keeps the last call's contents; every call rewrites what it reads, so no clearing is
 *     needed between calls.
 * Arguments, results and errors are otherwise those of plp_step. */
#define EGTP_STATIC_SCRATCH_BYTES (64u << 20)
size_t egtp_static_scratch_bytes(void);
egtp_status plp_step_static(egtp_ctx *ctx, const void *hidden_new, const int32_t *offsets_new_dev,
                            const int32_t *offsets_new_host, const int32_t *slot_dev, int32_t B,
                            int64_t T_new, float *pooled_state, float *lse_state, float *entropy_out,
                            float *rem_pred_out, void *stream);

/* Average / max / last-token pooling over the same ragged layout (Table 3's alternatives),
 * followed by head_len.  pooled_out [B x d] fp32, pred_out [B] fp32 (optional).  An empty
 * sequence pools to zeros. */
egtp_status egtp_pool_ablation(egtp_ctx *ctx, const void *hidden, const int32_t *offsets_dev,
                               const int32_t *offsets_host, int32_t B, int64_t T,
                               egtp_pool_kind kind, void *workspace, size_t workspace_bytes,
                               float *pooled_out, float *pred_out, void *stream);

/* Training of a K-bin head on frozen features (Section 3.2, 3.3; optimiser settings of the
 * experimental setup).  State of one head: fp32 parameters and their AdamW moments, all device
 * memory owned by the caller, all updated in place by egtp_head_train_step.  After training the
 * same w1/b1/w2/b2/bin_centers serve as an egtp_head with wdtype = EGTP_F32 and n_out = K. */
typedef struct {
    int32_t d;                /* feature size (multiple of 4) */
    int32_t d_h;              /* hidden width, 1 .. 16384 */
    int32_t K;                /* bins, 1 .. 1024 */
    float *w1, *b1;           /* [d_h x d], [d_h] */
    float *w2, *b2;           /* [K x d_h], [K] */
    float *m_w1, *v_w1;       /* first / second moment of each parameter, same shapes; zeros before */
    float *m_b1, *v_b1;       /* the first step */
    float *m_w2, *v_w2;
    float *m_b2, *v_b2;
    const float *bin_centers; /* [K], the c_i of Eq. 6 */
    float lambda;             /* weight of the cross-entropy term in Eq. 7, 0 .. 1 */
    float lr, beta1, beta2, eps, weight_decay; /* AdamW; lr >= 0, 0 <= beta < 1, eps > 0, decay >= 0 */
    int64_t t;                /* number of this step, 1 for the first (bias correction) */
    float *g_w1, *g_b1;       /* optional: receive the gradient of each parameter (NULL = not wanted) */
    float *g_w2, *g_b2;
} egtp_head_train;

/* Workspace bytes of one egtp_head_train_step with B samples; 0 if an argument is invalid. */
size_t egtp_head_train_workspace_bytes(int32_t B, int32_t d, int32_t d_h, int32_t K);

/* One optimisation step on B samples (x_b, bin_b, y_b):
 *   logits z_b = w2 relu(w1 x_b + b1) + b2,  phat_b = softmax(z_b),  yhat_b = sum_j phat_bj c_j  (Eq. 6)
 *   soft label p_bj = exp(-|j - bin_b|) / sum_k exp(-|k - bin_b|)                               (Eq. 5)
 *   loss = sum_b weight_b ( lambda CE(p_b, phat_b) + (1 - lambda) (y_b - yhat_b)^2 )             (Eq. 7)
 *   weight_b = 1/B, or, for PLP samples, 1 / (n_seqs * steps_per_seq[b]): the average over a
 *   sequence's decode steps, then over sequences                                               (Eq. 9)
 * followed by the gradient with respect to the four head parameters and one AdamW update
 *   m = beta1 m + (1-beta1) g,  v = beta2 v + (1-beta2) g^2,
 *   w = w - lr weight_decay w - lr (m / (1-beta1^t)) / (sqrt(v / (1-beta2^t)) + eps).
 *   x              [B x d] fp32 device: pooled vectors (egtp_score's pooled_out, a PLP state)
 *   bin            [B] int32 device: bin of the target, 0-based; values outside 0..K-1 are clamped.
 *                  The paper does not define the bin edges: the caller does the binning.
 *   y              [B] fp32 device: target length, in the unit of bin_centers
 *   steps_per_seq  [B] int32 device or NULL: for sample b, the number of decode steps (>= 1)
 *                  its sequence contributes to this batch; n_seqs = sequences in the batch
 *   loss_out       [3] fp32 device: the loss above, its CE sum and its MSE sum (before lambda)
 * Everything is enqueued on `stream`; nothing is allocated; fixed summation orders. */
egtp_status egtp_head_train_step(const egtp_head_train *head, const float *x, const int32_t *bin,
                                 const float *y, const int32_t *steps_per_seq, int32_t n_seqs, int32_t B,
                                 void *workspace, size_t workspace_bytes, float *loss_out, void *stream);

/* Diagnostic: how the fused LM-head + entropy kernel (Eq. 2) would be launched for T tokens --
 * one workgroup per (block of tokens_per_block tokens, range of tiles_per_range vocabulary tiles of
 * rows_per_tile rows); each leaves one partial (max, sum, weighted sum) triple per token, merged
 * afterwards.  paced = 1 when the kernel's workgroups keep each other in step (ranges longer
 * than four tiles, at least eight token blocks).  Pure host arithmetic: no device, no context.  Tests use it to make sure
 * that a shape reaches the launch configuration they mean to cover. */
typedef struct {
    int32_t tokens_per_block, rows_per_tile;
    int32_t token_blocks, vocab_tiles;
    int32_t vocab_ranges, tiles_per_range;
    int32_t paced;
} egtp_launch_plan;
egtp_status egtp_launch_plan_query(egtp_dtype dtype, int32_t d, int32_t vocab, int64_t T,
                                   egtp_launch_plan *out);

/* Measurement aid: when enabled, every egtp_score / plp_step call brackets its fused LM-head +
 * entropy kernel (the Eq. 2 contraction, where nearly all of the work is) with a pair of HIP
 * events on the call's stream.  The events are created here, not in the scoring calls; at most
 * `capacity` (<= 1024) calls are recorded until the next read.  on == 0 disables and frees. */
egtp_status egtp_profile_enable(egtp_ctx *ctx, int on, int capacity);
/* After the stream has been synchronised: writes the elapsed milliseconds of each recorded
 * kernel (oldest first) to ms_out[0..cap), returns how many were written and forgets them.
 * Returns -1 on error. */
int egtp_profile_read(egtp_ctx *ctx, float *ms_out_host, int cap);

/* Measurement aid: the rate the matrix cores sustain on this device when nothing else runs --
 * the reference the fused kernel's rate (Eq. 2 contraction) can be set against beside the
 * published peak.  Launches `launches` (1..64) kernels back to back on `stream`; each runs, on
 * 1024 workgroups of four waves, `iters` (1..10^7) steps of 64 bf16 MFMAs of the fused kernel's
 * shape on registers only, with all-zero operands (random_operands == 0: clock-limited) or
 * pseudo-random operands in [-1, 1) (power-limited).  Blocks until the last launch has ended.
 *   sink          device, >= egtp_mfma_probe_sink_floats() floats, overwritten
 *   tflops_out    host: [launches] achieved TFLOP/s of each launch (HIP events on `stream`)
 * Creates and destroys its events inside the call; allocates no device memory. */
size_t egtp_mfma_probe_sink_floats(void);
egtp_status egtp_mfma_probe(egtp_ctx *ctx, float *sink, size_t sink_floats, int32_t iters,
                            int32_t random_operands, int32_t launches, double *tflops_out_host,
                            void *stream);

/* Measurement aid: the rate at which this device streams a buffer out of HBM with plain 16-byte
 * loads and nothing else to do -- the reference the pooling kernels (Eq. 4 reads every hidden state
 * once more) can be set against beside the published bandwidth.  Launches `launches` (1..64) read
 * kernels over buf_dev[0 .. bytes) back to back on `stream` and blocks until the last has ended.
 *   buf_dev        device, 16-byte aligned, >= 1 MiB; only read.  Use a buffer much larger than the
 *                  caches (256 MiB of last-level cache on this part) or the figure is not HBM's
 *   sink_dev       device, >= egtp_hbm_read_probe_sink_bytes(), overwritten
 *   gbps_out_host  host: [launches] achieved GB/s (10^9 bytes per second) of each launch
 * Creates and destroys its events inside the call; allocates no device memory. */
size_t egtp_hbm_read_probe_sink_bytes(void);
egtp_status egtp_hbm_read_probe(egtp_ctx *ctx, const void *buf_dev, size_t bytes, void *sink_dev,
                                size_t sink_bytes, int32_t launches, double *gbps_out_host, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* EGTP_H */
