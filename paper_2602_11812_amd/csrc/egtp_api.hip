// C ABI of the EGTP / PLP library: argument checks, workspace carving, launch sequencing.
// Every arithmetic step runs in the kernels of this directory; nothing here computes.
#include "../../include/egtp.h"

#include <math.h>
#include <new>
#include <stdlib.h>
#include <string.h>

#include "kernels.h"

struct egtp_ctx {
    egtp_config cfg;
    int device;
    int last_hip_error;
    // optional event pairs around the fused entropy kernel (measurement aid)
    hipEvent_t *prof_events;  // 2 * prof_cap events, or NULL
    int prof_cap;
    int prof_count;
    // packed copy of W_lm for the matrix-core kernel (caller's memory), or NULL
    const void *w_packed;
    // this device's copy of the library's static scratch array (plp_step_static)
    void *static_scratch;
};

using namespace egtp;

// Scratch of plp_step_static: device memory that exists on every device the library is loaded on,
// from then until the process ends.  In host code this name only stands for the symbol; the
// address a kernel can use is looked up, for the device of each context, in egtp_create.
static __device__ __align__(256) unsigned char scratch[EGTP_STATIC_SCRATCH_BYTES];

namespace {

constexpr size_t ALIGN = 256;
inline size_t up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }

// Carves the caller's workspace; the same arithmetic gives egtp_workspace_bytes.
struct Carver {
    unsigned char *base;
    size_t off;
    explicit Carver(void *b) : base((unsigned char *)b), off(0) {}
    template <typename Tp>
    Tp *take(size_t count)
    {
        Tp *p = base ? (Tp *)(base + off) : nullptr;
        off += up(count * sizeof(Tp));
        return p;
    }
};

struct Workspace {
    float *entropy;      // [T]
    float *k1_part;      // partial triples
    int *k1_pace;        // pacing counters of the fused kernel
    int32_t *unit_start; // [B+1]
    float *lse_new;      // [B]
    float *state_scale;  // [B]
    float *pool_part;    // [units_bound x d]
    float *act;          // [k splits x B x d_h_max]
    unsigned char *hidden_packed;  // packed copy of this call's hidden states
    unsigned char *w_packed;       // when no persistent packed W_lm was given
    size_t bytes;
};

Workspace carve(const egtp_ctx *ctx, void *base, int64_t T, int32_t B)
{
    const egtp_config &c = ctx->cfg;
    Carver cv(base);
    Workspace w;
    // layer 1 leaves more planes when a head has fewer row tiles, so a narrower head can need more
    // floats than a wider one: the larger of the two bounds, not the bound of the larger width
    const size_t act_len = head_act_floats_bound(c.d, c.head_len.d_h, B, c.head_len.wdtype);
    const size_t act_rem = head_act_floats_bound(c.d, c.head_rem.d_h, B, c.head_rem.wdtype);
    w.entropy = cv.take<float>((size_t)T);
    w.k1_part = cv.take<float>(k1_partial_floats_bound(T));
    w.k1_pace = cv.take<int>(k1_pace_ints_bound(T));
    w.unit_start = cv.take<int32_t>((size_t)B + 1);
    w.lse_new = cv.take<float>((size_t)B);
    w.state_scale = cv.take<float>((size_t)B);
    w.pool_part = cv.take<float>((size_t)pool_units_bound(T, B) * (size_t)c.d);
    w.act = cv.take<float>(act_len > act_rem ? act_len : act_rem);
    const int K = (int)k1_contraction_len(c.dtype, c.d);
    w.hidden_packed = cv.take<unsigned char>(k1_packed_bytes(T, K));
    w.w_packed = ctx->w_packed ? nullptr : cv.take<unsigned char>(k1_packed_bytes(c.vocab, K));
    w.bytes = cv.off;
    return w;
}

egtp_status check_head(const egtp_head &h)
{
    if (h.d_h <= 0 || h.d_h > 16384 || h.n_out <= 0 || h.n_out > 1024)
        return EGTP_ERR_SHAPE;
    if (h.wdtype != EGTP_F32 && h.wdtype != EGTP_BF16)
        return EGTP_ERR_DTYPE;
    if (!h.w1 || !h.w2)
        return EGTP_ERR_NULL;
    if (h.n_out > 1 && !h.bin_centers)
        return EGTP_ERR_NULL;
    return EGTP_OK;
}

egtp_status check_offsets_host(const int32_t *o, int32_t B, int64_t T)
{
    if (o[0] != 0)
        return EGTP_ERR_OFFSETS;
    for (int32_t b = 0; b < B; ++b)
        if (o[b + 1] < o[b])
            return EGTP_ERR_OFFSETS;
    if ((int64_t)o[B] != T)
        return EGTP_ERR_OFFSETS;
    return EGTP_OK;
}

egtp_status hip_fail(egtp_ctx *ctx, hipError_t e)
{
    ctx->last_hip_error = (int)e;
    return EGTP_ERR_HIP;
}

#define EGTP_HIP(call)                \
    do {                              \
        hipError_t e_ = (call);       \
        if (e_ != hipSuccess)         \
            return hip_fail(ctx, e_); \
    } while (0)

// row-major operand -> the packed blocks the fused kernel reads (fp32: split into bf16 pieces on the way)
hipError_t pack_rows(int dtype, const void *src, int64_t rows, int d, bool hidden_side, void *dst, hipStream_t st)
{
    return dtype == EGTP_BF16 ? k1_pack_rows_bf16(src, rows, d, dst, st)
                              : k1_pack_rows_f32_split(src, rows, d, hidden_side, dst, st);
}

// Eq. 2 for T tokens: fused partials, then the per-token merge into `entropy` -- unless the caller merges
// them itself (nsplit_left != NULL receives the number of ranges still to be merged).
egtp_status run_entropy(egtp_ctx *ctx, const void *hidden, int64_t T, const Workspace &w, float *entropy,
                        hipStream_t st, int *nsplit_left = nullptr)
{
    const egtp_config &c = ctx->cfg;
    const K1Plan p = k1_plan(c.dtype, T, c.d, c.vocab);
    const bool timed = ctx->prof_events && ctx->prof_count < ctx->prof_cap;
    const void *wp = ctx->w_packed;
    if (!wp) {  // no persistent packed W_lm: pack it for this call
        EGTP_HIP(pack_rows(c.dtype, c.w_lm, c.vocab, c.d, false, w.w_packed, st));
        wp = w.w_packed;
    }
    EGTP_HIP(pack_rows(c.dtype, hidden, T, c.d, true, w.hidden_packed, st));
    if (timed)
        EGTP_HIP(hipEventRecord(ctx->prof_events[2 * ctx->prof_count], st));
    EGTP_HIP(k1_entropy_bf16(w.hidden_packed, wp, T, (int)k1_contraction_len(c.dtype, c.d), c.vocab, p, w.k1_part,
                             w.k1_pace, st));
    if (timed) {
        EGTP_HIP(hipEventRecord(ctx->prof_events[2 * ctx->prof_count + 1], st));
        ++ctx->prof_count;
    }
    if (nsplit_left)
        *nsplit_left = p.nsplit;
    else
        EGTP_HIP(k1_merge(w.k1_part, p.nsplit, T, entropy, st));
    return EGTP_OK;
}

egtp_status run_head(egtp_ctx *ctx, const egtp_head &h, const float *x, const int32_t *slot, int32_t B,
                     const Workspace &w, float *pred, float *p_hat, hipStream_t st)
{
    HeadArgs a;
    a.p_hat = p_hat;
    a.x = x;
    a.slot = slot;
    a.B = B;
    a.d = ctx->cfg.d;
    a.d_h = h.d_h;
    a.n_out = h.n_out;
    a.wdtype = h.wdtype;
    a.w1 = h.w1;
    a.b1 = h.b1;
    a.w2 = h.w2;
    a.b2 = h.b2;
    a.bin_centers = h.bin_centers;
    a.act = w.act;
    a.pred = pred;
    EGTP_HIP(head_forward(a, st));
    return EGTP_OK;
}

egtp_status check_common(const egtp_ctx *ctx, int32_t B, int64_t T, const void *workspace, size_t ws_bytes)
{
    if (!ctx)
        return EGTP_ERR_NULL;
    if (B < 0 || T < 0 || T > 0x7fffffffLL)
        return EGTP_ERR_SHAPE;
    if (B == 0 && T != 0)
        return EGTP_ERR_SHAPE;
    if (B > 0) {
        if (!workspace || ((uintptr_t)workspace % ALIGN) != 0)
            return EGTP_ERR_WORKSPACE;
        if (ws_bytes < egtp_workspace_bytes(ctx, T, B))
            return EGTP_ERR_WORKSPACE;
    }
    return EGTP_OK;
}

}  // namespace

extern "C" {

const char *egtp_status_string(egtp_status s)
{
    switch (s) {
    case EGTP_OK: return "ok";
    case EGTP_ERR_NULL: return "a required pointer is NULL";
    case EGTP_ERR_SHAPE: return "invalid or unsupported size";
    case EGTP_ERR_OFFSETS: return "malformed offsets";
    case EGTP_ERR_DTYPE: return "unknown storage type";
    case EGTP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case EGTP_ERR_ARCH: return "current device is not gfx950";
    case EGTP_ERR_HIP: return "HIP call failed";
    case EGTP_ERR_ALPHA: return "temperature must be finite and > 0";
    case EGTP_ERR_HYPER: return "training hyper-parameter out of range";
    }
    return "unknown status";
}

egtp_status egtp_create(const egtp_config *cfg, egtp_ctx **out)
{
    if (!cfg || !out)
        return EGTP_ERR_NULL;
    if (cfg->dtype != EGTP_F32 && cfg->dtype != EGTP_BF16)
        return EGTP_ERR_DTYPE;
    if (cfg->d <= 0 || cfg->vocab <= 0)
        return EGTP_ERR_SHAPE;
    if (cfg->d % (cfg->dtype == EGTP_BF16 ? 8 : 4) != 0)
        return EGTP_ERR_SHAPE;  // rows must start on 16-byte boundaries
    if (k1_contraction_len(cfg->dtype, cfg->d) > K1_MAX_CONTRACTION)
        return EGTP_ERR_SHAPE;  // the fused kernel addresses a packed row tile over all of K with 32-bit byte offsets
    if (!(cfg->alpha > 0.0f) || !isfinite(cfg->alpha))
        return EGTP_ERR_ALPHA;
    egtp_status s = check_head(cfg->head_len);
    if (s != EGTP_OK)
        return s;
    if (cfg->head_rem.w1) {
        s = check_head(cfg->head_rem);
        if (s != EGTP_OK)
            return s;
    }
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess)
        return EGTP_ERR_ARCH;
    hipDeviceProp_t prop;
    e = hipGetDeviceProperties(&prop, dev);
    if (e != hipSuccess || strncmp(prop.gcnArchName, "gfx950", 6) != 0)
        return EGTP_ERR_ARCH;
    egtp_ctx *ctx = new (std::nothrow) egtp_ctx;
    if (!ctx)
        return EGTP_ERR_HIP;
    ctx->cfg = *cfg;
    if (!cfg->head_rem.w1)
        ctx->cfg.head_rem = cfg->head_len;
    ctx->device = dev;
    ctx->last_hip_error = 0;
    ctx->prof_events = nullptr;
    ctx->prof_cap = 0;
    ctx->prof_count = 0;
    ctx->w_packed = nullptr;
    ctx->static_scratch = nullptr;
    // this device's address of the static scratch array (the device is current here)
    e = hipGetSymbolAddress(&ctx->static_scratch, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ctx->static_scratch) {
        delete ctx;
        return EGTP_ERR_HIP;
    }
    *out = ctx;
    return EGTP_OK;
}

static void free_profile(egtp_ctx *ctx)
{
    if (ctx->prof_events) {
        for (int i = 0; i < 2 * ctx->prof_cap; ++i)
            if (ctx->prof_events[i])
                (void)hipEventDestroy(ctx->prof_events[i]);
        delete[] ctx->prof_events;
    }
    ctx->prof_events = nullptr;
    ctx->prof_cap = 0;
    ctx->prof_count = 0;
}

egtp_status egtp_destroy(egtp_ctx *ctx)
{
    if (ctx)
        free_profile(ctx);
    delete ctx;
    return EGTP_OK;
}

egtp_status egtp_profile_enable(egtp_ctx *ctx, int on, int capacity)
{
    if (!ctx)
        return EGTP_ERR_NULL;
    free_profile(ctx);
    if (!on)
        return EGTP_OK;
    if (capacity <= 0 || capacity > 1024)
        return EGTP_ERR_SHAPE;
    ctx->prof_events = new (std::nothrow) hipEvent_t[2 * capacity]();
    if (!ctx->prof_events)
        return EGTP_ERR_HIP;
    ctx->prof_cap = capacity;
    for (int i = 0; i < 2 * capacity; ++i) {
        hipError_t e = hipEventCreate(&ctx->prof_events[i]);
        if (e != hipSuccess) {
            ctx->prof_events[i] = nullptr;
            free_profile(ctx);
            return hip_fail(ctx, e);
        }
    }
    return EGTP_OK;
}

int egtp_profile_read(egtp_ctx *ctx, float *ms_out_host, int cap)
{
    if (!ctx || !ms_out_host || cap < 0)
        return -1;
    int n = ctx->prof_count < cap ? ctx->prof_count : cap;
    for (int i = 0; i < n; ++i) {
        hipError_t e = hipEventElapsedTime(&ms_out_host[i], ctx->prof_events[2 * i], ctx->prof_events[2 * i + 1]);
        if (e != hipSuccess) {
            ctx->last_hip_error = (int)e;
            return -1;
        }
    }
    ctx->prof_count = 0;
    return n;
}

size_t egtp_mfma_probe_sink_floats(void) { return (size_t)MFMA_PROBE_WORKGROUPS * 256; }

egtp_status egtp_mfma_probe(egtp_ctx *ctx, float *sink, size_t sink_floats, int32_t iters,
                            int32_t random_operands, int32_t launches, double *tflops_out_host,
                            void *stream)
{
    if (!ctx || !sink || !tflops_out_host)
        return EGTP_ERR_NULL;
    if (iters < 1 || iters > 10000000 || launches < 1 || launches > 64)
        return EGTP_ERR_SHAPE;
    if (sink_floats < egtp_mfma_probe_sink_floats())
        return EGTP_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t ev[65] = {};
    hipError_t e = hipSuccess;
    for (int i = 0; i <= launches && e == hipSuccess; ++i)
        e = hipEventCreate(&ev[i]);
    if (e == hipSuccess)
        e = hipEventRecord(ev[0], st);
    for (int i = 0; i < launches && e == hipSuccess; ++i) {
        e = mfma_probe_launch(sink, iters, random_operands != 0, st);
        if (e == hipSuccess)
            e = hipEventRecord(ev[i + 1], st);
    }
    if (e == hipSuccess)
        e = hipEventSynchronize(ev[launches]);
    for (int i = 0; i < launches && e == hipSuccess; ++i) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, ev[i], ev[i + 1]);
        tflops_out_host[i] = ms > 0.f ? mfma_probe_flop(iters) / ((double)ms * 1e-3) / 1e12 : 0.0;
    }
    for (int i = 0; i <= launches; ++i)
        if (ev[i])
            (void)hipEventDestroy(ev[i]);
    return e == hipSuccess ? EGTP_OK : hip_fail(ctx, e);
}

egtp_status egtp_launch_plan_query(egtp_dtype dtype, int32_t d, int32_t vocab, int64_t T, egtp_launch_plan *out)
{
    if (!out)
        return EGTP_ERR_NULL;
    if (dtype != EGTP_F32 && dtype != EGTP_BF16)
        return EGTP_ERR_DTYPE;
    if (d <= 0 || vocab <= 0 || T < 0 || T > 0x7fffffffLL)
        return EGTP_ERR_SHAPE;
    const K1Plan p = k1_plan(dtype, T, d, vocab);
    out->tokens_per_block = p.tb_tokens;
    out->rows_per_tile = p.tile_v;
    out->token_blocks = p.ntb;
    out->vocab_tiles = p.ntiles_v;
    out->vocab_ranges = p.nsplit;
    out->tiles_per_range = p.tiles_per_split;
    out->paced = T > 0 && k1_plan_paces(p) ? 1 : 0;
    return EGTP_OK;
}

size_t egtp_hbm_read_probe_sink_bytes(void) { return (size_t)HBM_PROBE_WORKGROUPS * 256 * sizeof(unsigned); }

egtp_status egtp_hbm_read_probe(egtp_ctx *ctx, const void *buf_dev, size_t bytes, void *sink_dev, size_t sink_bytes,
                                int32_t launches, double *gbps_out_host, void *stream)
{
    if (!ctx || !buf_dev || !sink_dev || !gbps_out_host)
        return EGTP_ERR_NULL;
    if (launches < 1 || launches > 64 || bytes < ((size_t)1 << 20) || ((uintptr_t)buf_dev % 16) != 0)
        return EGTP_ERR_SHAPE;
    if (sink_bytes < egtp_hbm_read_probe_sink_bytes() || ((uintptr_t)sink_dev % 4) != 0)
        return EGTP_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    hipEvent_t ev[65] = {};
    hipError_t e = hipSuccess;
    for (int i = 0; i <= launches && e == hipSuccess; ++i)
        e = hipEventCreate(&ev[i]);
    if (e == hipSuccess)
        e = hipEventRecord(ev[0], st);
    for (int i = 0; i < launches && e == hipSuccess; ++i) {
        e = hbm_read_probe_launch(buf_dev, bytes, (unsigned *)sink_dev, st);
        if (e == hipSuccess)
            e = hipEventRecord(ev[i + 1], st);
    }
    if (e == hipSuccess)
        e = hipEventSynchronize(ev[launches]);
    for (int i = 0; i < launches && e == hipSuccess; ++i) {
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, ev[i], ev[i + 1]);
        gbps_out_host[i] = ms > 0.f ? (double)(bytes / 16 * 16) / ((double)ms * 1e-3) / 1e9 : 0.0;
    }
    for (int i = 0; i <= launches; ++i)
        if (ev[i])
            (void)hipEventDestroy(ev[i]);
    return e == hipSuccess ? EGTP_OK : hip_fail(ctx, e);
}

size_t egtp_workspace_bytes(const egtp_ctx *ctx, int64_t max_tokens, int32_t max_seqs)
{
    if (!ctx || max_tokens < 0 || max_seqs < 0 || max_tokens > 0x7fffffffLL)
        return 0;
    return carve(ctx, nullptr, max_tokens, max_seqs).bytes;
}

int egtp_last_hip_error(const egtp_ctx *ctx) { return ctx ? ctx->last_hip_error : 0; }

size_t egtp_packed_w_lm_bytes(const egtp_ctx *ctx)
{
    if (!ctx)
        return 0;
    return k1_packed_bytes(ctx->cfg.vocab, (int)k1_contraction_len(ctx->cfg.dtype, ctx->cfg.d));
}

egtp_status egtp_pack_w_lm(egtp_ctx *ctx, void *packed_dev, size_t bytes, void *stream)
{
    if (!ctx)
        return EGTP_ERR_NULL;
    if (!packed_dev) {  // forget the packed copy
        ctx->w_packed = nullptr;
        return EGTP_OK;
    }
    if (!ctx->cfg.w_lm)
        return EGTP_ERR_NULL;  // nothing to pack from
    if (((uintptr_t)packed_dev % ALIGN) != 0 || bytes < egtp_packed_w_lm_bytes(ctx))
        return EGTP_ERR_WORKSPACE;
    EGTP_HIP(pack_rows(ctx->cfg.dtype, ctx->cfg.w_lm, ctx->cfg.vocab, ctx->cfg.d, false, packed_dev,
                       (hipStream_t)stream));
    ctx->w_packed = packed_dev;
    return EGTP_OK;
}

egtp_status egtp_adopt_packed_w_lm(egtp_ctx *ctx, const void *packed_dev, size_t bytes)
{
    if (!ctx || !packed_dev)
        return EGTP_ERR_NULL;
    if (((uintptr_t)packed_dev % ALIGN) != 0 || bytes < egtp_packed_w_lm_bytes(ctx))
        return EGTP_ERR_WORKSPACE;
    ctx->w_packed = packed_dev;
    return EGTP_OK;
}

size_t egtp_static_scratch_bytes(void) { return (size_t)EGTP_STATIC_SCRATCH_BYTES; }

egtp_status egtp_build_offsets(egtp_ctx *ctx, const int32_t *lengths_dev, int32_t B, int32_t *offsets_dev,
                               int32_t *seg_ids_dev, int64_t T, void *stream)
{
    if (!ctx || !offsets_dev || (B > 0 && !lengths_dev))
        return EGTP_ERR_NULL;
    if (B < 0 || T < 0 || T > 0x7fffffffLL)
        return EGTP_ERR_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    EGTP_HIP(scan_lengths(lengths_dev, B, offsets_dev, st));
    if (seg_ids_dev && T > 0)
        EGTP_HIP(segment_ids(offsets_dev, B, T, seg_ids_dev, st));
    return EGTP_OK;
}

}  // extern "C"

namespace {

// a context without the row-major W_lm can only score from a packed copy
bool lm_head_missing(const egtp_ctx *ctx) { return !ctx->cfg.w_lm && !ctx->w_packed; }

egtp_status score_impl(egtp_ctx *ctx, const void *hidden, const int32_t *offsets_dev,
                       const int32_t *offsets_host, int32_t B, int64_t T, void *workspace,
                       size_t workspace_bytes, float *entropy_out, float *pooled_out, float *lse_out,
                       float *pred_out, float *p_hat_out, bool want_p_hat, void *stream)
{
    egtp_status s = check_common(ctx, B, T, workspace, workspace_bytes);
    if (s != EGTP_OK)
        return s;
    if (want_p_hat && ctx->cfg.head_len.n_out < 2)
        return EGTP_ERR_SHAPE;  // a scalar head has no distribution
    if (B == 0)
        return EGTP_OK;
    if (!offsets_dev || !pooled_out || !lse_out || !pred_out || (T > 0 && !hidden) || (want_p_hat && !p_hat_out))
        return EGTP_ERR_NULL;
    if (T > 0 && lm_head_missing(ctx))
        return EGTP_ERR_NULL;
    if (offsets_host && (s = check_offsets_host(offsets_host, B, T)) != EGTP_OK)
        return s;

    hipStream_t st = (hipStream_t)stream;
    const egtp_config &c = ctx->cfg;
    const Workspace w = carve(ctx, workspace, T, B);
    float *entropy = entropy_out ? entropy_out : w.entropy;
    if (T > 0 && (s = run_entropy(ctx, hidden, T, w, entropy, st)) != EGTP_OK)
        return s;

    PoolArgs a;
    a.hidden = hidden;
    a.dtype = c.dtype;
    a.d = c.d;
    a.entropy = entropy;
    a.k1_part = nullptr;
    a.k1_nsplit = 0;
    a.offsets = offsets_dev;
    a.slot = nullptr;
    a.B = B;
    a.T = T;
    a.inv_alpha = 1.0f / c.alpha;
    a.state_lse = nullptr;
    a.state_pooled = nullptr;
    a.out_pooled = pooled_out;
    a.out_lse = lse_out;
    a.unit_start = w.unit_start;
    a.lse_new = w.lse_new;
    a.state_scale = w.state_scale;
    a.partial = w.pool_part;
    EGTP_HIP(pool_entropy_weighted(a, st));
    return run_head(ctx, c.head_len, pooled_out, nullptr, B, w, pred_out, p_hat_out, st);
}

egtp_status step_impl(egtp_ctx *ctx, const void *hidden_new, const int32_t *offsets_new_dev,
                      const int32_t *offsets_new_host, const int32_t *slot_dev, int32_t B, int64_t T_new,
                      float *pooled_state, float *lse_state, void *workspace, size_t workspace_bytes,
                      float *entropy_out, float *rem_pred_out, float *p_hat_out, bool want_p_hat, void *stream)
{
    egtp_status s = check_common(ctx, B, T_new, workspace, workspace_bytes);
    if (s != EGTP_OK)
        return s;
    if (want_p_hat && ctx->cfg.head_rem.n_out < 2)
        return EGTP_ERR_SHAPE;
    if (B == 0)
        return EGTP_OK;
    if (!pooled_state || !lse_state || !rem_pred_out || (T_new > 0 && !hidden_new) || (want_p_hat && !p_hat_out))
        return EGTP_ERR_NULL;
    if (T_new > 0 && lm_head_missing(ctx))
        return EGTP_ERR_NULL;
    if (!offsets_new_dev) {
        if (T_new != B)
            return EGTP_ERR_SHAPE;
        if (offsets_new_host)
            return EGTP_ERR_OFFSETS;  // a host mirror of offsets that were not given
    } else if (offsets_new_host && (s = check_offsets_host(offsets_new_host, B, T_new)) != EGTP_OK) {
        return s;
    }

    hipStream_t st = (hipStream_t)stream;
    const egtp_config &c = ctx->cfg;
    const Workspace w = carve(ctx, workspace, T_new, B);
    float *entropy = entropy_out ? entropy_out : w.entropy;
    // one token per sequence: the state update finishes the entropy itself (one launch less per decode step)
    int nsplit_left = 0;
    if (T_new > 0 &&
        (s = run_entropy(ctx, hidden_new, T_new, w, entropy, st, offsets_new_dev ? nullptr : &nsplit_left)) != EGTP_OK)
        return s;

    PoolArgs a;
    a.hidden = hidden_new;
    a.dtype = c.dtype;
    a.d = c.d;
    a.entropy = entropy;
    a.k1_part = nsplit_left > 0 ? w.k1_part : nullptr;
    a.k1_nsplit = nsplit_left;
    a.offsets = offsets_new_dev;
    a.slot = slot_dev;
    a.B = B;
    a.T = T_new;
    a.inv_alpha = 1.0f / c.alpha;
    a.state_lse = lse_state;
    a.state_pooled = pooled_state;
    a.out_pooled = pooled_state;
    a.out_lse = lse_state;
    a.unit_start = w.unit_start;
    a.lse_new = w.lse_new;
    a.state_scale = w.state_scale;
    a.partial = w.pool_part;
    EGTP_HIP(pool_entropy_weighted(a, st));
    return run_head(ctx, c.head_rem, pooled_state, slot_dev, B, w, rem_pred_out, p_hat_out, st);
}

}  // namespace

extern "C" {

egtp_status egtp_score(egtp_ctx *ctx, const void *hidden, const int32_t *offsets_dev,
                       const int32_t *offsets_host, int32_t B, int64_t T, void *workspace,
                       size_t workspace_bytes, float *entropy_out, float *pooled_out, float *lse_out,
                       float *pred_out, void *stream)
{
    return score_impl(ctx, hidden, offsets_dev, offsets_host, B, T, workspace, workspace_bytes, entropy_out,
                      pooled_out, lse_out, pred_out, nullptr, false, stream);
}

egtp_status egtp_score_dist(egtp_ctx *ctx, const void *hidden, const int32_t *offsets_dev,
                            const int32_t *offsets_host, int32_t B, int64_t T, void *workspace,
                            size_t workspace_bytes, float *entropy_out, float *pooled_out, float *lse_out,
                            float *pred_out, float *p_hat_out, void *stream)
{
    return score_impl(ctx, hidden, offsets_dev, offsets_host, B, T, workspace, workspace_bytes, entropy_out,
                      pooled_out, lse_out, pred_out, p_hat_out, true, stream);
}

egtp_status plp_step(egtp_ctx *ctx, const void *hidden_new, const int32_t *offsets_new_dev,
                     const int32_t *offsets_new_host, const int32_t *slot_dev, int32_t B, int64_t T_new,
                     float *pooled_state, float *lse_state, void *workspace, size_t workspace_bytes,
                     float *entropy_out, float *rem_pred_out, void *stream)
{
    return step_impl(ctx, hidden_new, offsets_new_dev, offsets_new_host, slot_dev, B, T_new, pooled_state,
                     lse_state, workspace, workspace_bytes, entropy_out, rem_pred_out, nullptr, false, stream);
}

egtp_status plp_step_dist(egtp_ctx *ctx, const void *hidden_new, const int32_t *offsets_new_dev,
                          const int32_t *offsets_new_host, const int32_t *slot_dev, int32_t B, int64_t T_new,
                          float *pooled_state, float *lse_state, void *workspace, size_t workspace_bytes,
                          float *entropy_out, float *rem_pred_out, float *p_hat_out, void *stream)
{
    return step_impl(ctx, hidden_new, offsets_new_dev, offsets_new_host, slot_dev, B, T_new, pooled_state,
                     lse_state, workspace, workspace_bytes, entropy_out, rem_pred_out, p_hat_out, true, stream);
}

egtp_status plp_step_static(egtp_ctx *ctx, const void *hidden_new, const int32_t *offsets_new_dev,
                            const int32_t *offsets_new_host, const int32_t *slot_dev, int32_t B, int64_t T_new,
                            float *pooled_state, float *lse_state, float *entropy_out, float *rem_pred_out,
                            void *stream)
{
    if (!ctx)
        return EGTP_ERR_NULL;
    if (B < 0 || T_new < 0 || T_new > 0x7fffffffLL)
        return EGTP_ERR_SHAPE;
    // the scratch array is this call's whole workspace: larger batches are the caller's to split
    const size_t need = egtp_workspace_bytes(ctx, T_new, B);
    if (need > (size_t)EGTP_STATIC_SCRATCH_BYTES)
        return EGTP_ERR_WORKSPACE;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev != ctx->device)
        return EGTP_ERR_ARCH;  // the array's address was looked up for the context's device
    return step_impl(ctx, hidden_new, offsets_new_dev, offsets_new_host, slot_dev, B, T_new, pooled_state,
                     lse_state, ctx->static_scratch, (size_t)EGTP_STATIC_SCRATCH_BYTES, entropy_out,
                     rem_pred_out, nullptr, false, stream);
}

egtp_status egtp_pool_ablation(egtp_ctx *ctx, const void *hidden, const int32_t *offsets_dev,
                               const int32_t *offsets_host, int32_t B, int64_t T, egtp_pool_kind kind,
                               void *workspace, size_t workspace_bytes, float *pooled_out, float *pred_out,
                               void *stream)
{
    egtp_status s = check_common(ctx, B, T, workspace, workspace_bytes);
    if (s != EGTP_OK)
        return s;
    if (kind != EGTP_POOL_AVERAGE && kind != EGTP_POOL_MAX && kind != EGTP_POOL_LAST)
        return EGTP_ERR_SHAPE;
    if (B == 0)
        return EGTP_OK;
    if (!offsets_dev || !pooled_out || (T > 0 && !hidden))
        return EGTP_ERR_NULL;
    if (offsets_host && (s = check_offsets_host(offsets_host, B, T)) != EGTP_OK)
        return s;
    hipStream_t st = (hipStream_t)stream;
    const egtp_config &c = ctx->cfg;
    const Workspace w = carve(ctx, workspace, T, B);
    EGTP_HIP(pool_plain(hidden, c.dtype, c.d, offsets_dev, B, T, (int)kind, w.unit_start, w.pool_part, pooled_out,
                        st));
    if (pred_out)
        return run_head(ctx, c.head_len, pooled_out, nullptr, B, w, pred_out, nullptr, st);
    return EGTP_OK;
}

// ---- head training ----------------------------------------------------------------------------
namespace {

struct TrainWorkspace {
    float *act_part, *act, *dact, *dz, *loss_part;
    size_t bytes;
};

TrainWorkspace carve_train(void *base, int32_t B, int32_t d, int32_t d_h, int32_t K)
{
    Carver cv(base);
    TrainWorkspace w;
    w.act_part = cv.take<float>(head_act_floats_bound(d, d_h, B, DT_F32));
    w.act = cv.take<float>((size_t)B * (size_t)d_h);
    w.dact = cv.take<float>((size_t)B * (size_t)d_h);
    w.dz = cv.take<float>((size_t)B * (size_t)K);
    w.loss_part = cv.take<float>((size_t)B * 2);
    w.bytes = cv.off;
    return w;
}

bool train_shape_ok(int32_t B, int32_t d, int32_t d_h, int32_t K)
{
    return B >= 0 && d > 0 && d % 4 == 0 && d_h > 0 && d_h <= 16384 && K > 0 && K <= 1024;
}

}  // namespace

size_t egtp_head_train_workspace_bytes(int32_t B, int32_t d, int32_t d_h, int32_t K)
{
    if (!train_shape_ok(B, d, d_h, K))
        return 0;
    return carve_train(nullptr, B, d, d_h, K).bytes;
}

egtp_status egtp_head_train_step(const egtp_head_train *h, const float *x, const int32_t *bin, const float *y,
                                 const int32_t *steps_per_seq, int32_t n_seqs, int32_t B, void *workspace,
                                 size_t workspace_bytes, float *loss_out, void *stream)
{
    if (!h)
        return EGTP_ERR_NULL;
    if (!train_shape_ok(B, h->d, h->d_h, h->K))
        return EGTP_ERR_SHAPE;
    if (!h->w1 || !h->b1 || !h->w2 || !h->b2 || !h->m_w1 || !h->v_w1 || !h->m_b1 || !h->v_b1 || !h->m_w2 ||
        !h->v_w2 || !h->m_b2 || !h->v_b2 || !h->bin_centers)
        return EGTP_ERR_NULL;
    if (!(h->lambda >= 0.0f && h->lambda <= 1.0f) || !(h->lr >= 0.0f) || !isfinite(h->lr) ||
        !(h->beta1 >= 0.0f && h->beta1 < 1.0f) || !(h->beta2 >= 0.0f && h->beta2 < 1.0f) || !(h->eps > 0.0f) ||
        !isfinite(h->eps) || !(h->weight_decay >= 0.0f) || !isfinite(h->weight_decay) || h->t < 1)
        return EGTP_ERR_HYPER;
    if (B == 0)
        return EGTP_OK;
    if (!x || !bin || !y || !loss_out)
        return EGTP_ERR_NULL;
    if (steps_per_seq && n_seqs <= 0)
        return EGTP_ERR_SHAPE;
    if (!workspace || ((uintptr_t)workspace % ALIGN) != 0 ||
        workspace_bytes < egtp_head_train_workspace_bytes(B, h->d, h->d_h, h->K))
        return EGTP_ERR_WORKSPACE;
    // the architecture check is remembered per device: this call is made once per training step
    static DeviceMask arch_checked{0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess)
        return EGTP_ERR_ARCH;
    if (!device_bit_set(arch_checked, dev)) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, dev) != hipSuccess || strncmp(prop.gcnArchName, "gfx950", 6) != 0)
            return EGTP_ERR_ARCH;
        set_device_bit(arch_checked, dev);
    }

    const TrainWorkspace w = carve_train(workspace, B, h->d, h->d_h, h->K);
    TrainArgs a;
    a.x = x;
    a.bin = bin;
    a.y = y;
    a.steps = steps_per_seq;
    a.n_seqs = n_seqs;
    a.B = B;
    a.d = h->d;
    a.d_h = h->d_h;
    a.K = h->K;
    a.w1 = h->w1, a.b1 = h->b1, a.w2 = h->w2, a.b2 = h->b2;
    a.m_w1 = h->m_w1, a.v_w1 = h->v_w1, a.m_b1 = h->m_b1, a.v_b1 = h->v_b1;
    a.m_w2 = h->m_w2, a.v_w2 = h->v_w2, a.m_b2 = h->m_b2, a.v_b2 = h->v_b2;
    a.centers = h->bin_centers;
    a.lambda = h->lambda;
    a.lr = h->lr;
    a.beta1 = h->beta1;
    a.beta2 = h->beta2;
    a.eps = h->eps;
    a.weight_decay = h->weight_decay;
    // scalar factors of the update, formed once in double
    a.omb1 = (float)(1.0 - (double)h->beta1);
    a.omb2 = (float)(1.0 - (double)h->beta2);
    a.corr1 = (float)(1.0 - pow((double)h->beta1, (double)h->t));
    a.corr2 = (float)(1.0 - pow((double)h->beta2, (double)h->t));
    a.g_w1 = h->g_w1, a.g_b1 = h->g_b1, a.g_w2 = h->g_w2, a.g_b2 = h->g_b2;
    a.loss = loss_out;
    a.act_part = w.act_part;
    a.act = w.act;
    a.dact = w.dact;
    a.dz = w.dz;
    a.loss_part = w.loss_part;
    return head_train_step(a, (hipStream_t)stream) == hipSuccess ? EGTP_OK : EGTP_ERR_HIP;
}

}  // extern "C"
