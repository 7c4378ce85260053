/*
 * tokfilt.h - C ABI of the MI355X (gfx950) Token Filtering hot path.
 *
 * One attention layer of the method of arxiv 2512.07090 ("Leveraging KV Similarity for Online
 * Structured Pruning in LLMs"): every token is scored by the per-head cosine similarity of
 * its key and value with the mean of all previous keys and values (Algorithm 1, Section 3.2),
 * the two similarities are fused across heads with the variance-aware weight of Eq. 2, the
 * most redundant tokens are filtered at a target ratio, and causal attention runs over the
 * kept tokens only, filtered tokens receiving a zero attention output (Section 3.2).
 *
 * Groups of entry points
 *   - batched, exact count:  tf_score, tf_select, tf_attend, tf_filtered_attention
 *     (tf_filtered_attention_static: the same without a workspace argument)
 *   - batched, online threshold (Section 3.3, Eq. 4):  tf_select_online, tf_attend_ragged,
 *     tf_filtered_attention_online
 *   - tail-focused layer schedule (Eq. 3):  tf_tail_schedule, tf_filtered_attention_layers
 *   - one token at a time with caller-held state (Algorithm 1 as a call per token):
 *     tf_decode_init, tf_decode_prefill, tf_decode_step
 *   - measurement:  tf_stage_timing_*, tf_probe_*
 * Variants selected through tf_params: the incremental anchor of Eq. 1 (anchor, ema_gamma), the
 * anchor that includes the current token (anchor_inclusive), key-only / value-only scores and
 * the two readings of Eq. 2 (fusion).
 *
 * Conventions for every entry point
 *   - Pointers named Q, K, V, O, fused, sim_k, sim_v, keep, kept_idx, tau and ws are DEVICE
 *     pointers on the context's GPU.  `tf_params` and everything else is HOST memory.
 *   - Layout: Q and O are [batch][n_q_heads][seq][head_dim], K and V are
 *     [batch][n_kv_heads][seq][head_dim]; head_dim is contiguous; the other three extents
 *     use the element strides given in tf_params (so [batch][seq][head][dim] storage works).
 *     Base pointers must be 16-byte aligned and strides multiples of 8 elements.
 *   - Ownership: the caller owns every buffer, including the workspace; the library
 *     allocates no device memory in these calls and keeps no pointer after returning.
 *   - Ordering: work is enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and the call returns without waiting.  Outputs are valid once the
 *     caller has synchronised the stream.
 *   - Errors: a tf_status is returned, nothing is thrown.  Argument errors are found on
 *     the host before anything is enqueued and leave all outputs untouched; tf_last_error
 *     gives a sentence describing the most recent failure on that context.
 *   - NaN or infinite inputs: behaviour unspecified.
 */
#ifndef TOKFILT_H
#define TOKFILT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct tf_ctx tf_ctx; /* opaque: device id, timing events */

typedef enum {
    TF_OK = 0,
    TF_ERR_INVALID_ARG = 1,
    TF_ERR_UNSUPPORTED = 2,
    TF_ERR_WORKSPACE_TOO_SMALL = 3,
    TF_ERR_DEVICE = 4
} tf_status;

typedef enum { TF_F32 = 0, TF_BF16 = 1 } tf_dtype;

/* How the key and value similarities are combined (Eq. 2 / Algorithm 1).
 *   TF_FUSE_EQ2     alpha = sigma_v^-2 / (sigma_k^-2 + sigma_v^-2), exactly as printed;
 *   TF_FUSE_INVVAR  alpha = sigma_k^-2 / (sigma_k^-2 + sigma_v^-2), the weighting the prose
 *                   describes (more weight on the lower-variance side);
 *   TF_FUSE_KEY_ONLY / TF_FUSE_VALUE_ONLY  alpha = 1 / alpha = 0 (the ablation of Table 7).
 * S = alpha * s_k + (1 - alpha) * s_v, where s and sigma^2 are the mean and population
 * variance over KV heads of one token's cosines; 1e-12 is added to each variance. */
typedef enum {
    TF_FUSE_EQ2 = 0,
    TF_FUSE_INVVAR = 1,
    TF_FUSE_KEY_ONLY = 2,
    TF_FUSE_VALUE_ONLY = 3
} tf_fusion;

/* The anchor a token's key / value is compared with.
 * TF_ANCHOR_MEAN  the exact mean of all previous rows (Algorithm 1, Section 3.2).
 * TF_ANCHOR_EMA   the incremental anchor of Eq. 1: Anchor <- gamma * Anchor +
 *                 (1 - gamma) * row, starting from zero; a row is compared with the anchor as
 *                 it stands before that row is folded in. */
typedef enum { TF_ANCHOR_MEAN = 0, TF_ANCHOR_EMA = 1 } tf_anchor;

typedef struct {
    int32_t batch;         /* 1 .. 65535 */
    int32_t n_q_heads;     /* 1 .. 65535 */
    int32_t n_kv_heads;    /* n_q_heads % n_kv_heads == 0 (grouped-query attention) */
    int32_t seq;           /* n >= 1 */
    int32_t head_dim;      /* only 128 is supported */
    int32_t dtype;         /* tf_dtype of Q, K, V and O */
    int64_t q_stride[3];   /* element strides of Q for (batch, head, position) */
    int64_t kv_stride[3];  /* element strides shared by K and V */
    int64_t o_stride[3];   /* element strides of O */
    double prune_ratio;    /* r in [0, 1): fraction of tokens filtered */
    int32_t warmup;        /* W >= 0: the first min(W, m) tokens are always kept (warm-up
                              phase of Section 3.2); 1 is the usual value, token 0 has no
                              anchor */
    int32_t fusion;        /* tf_fusion */
    float softmax_scale;   /* 0 means 1 / sqrt(head_dim) */
    int32_t anchor;        /* tf_anchor; 0 (the exact mean) is the default */
    float ema_gamma;       /* smoothing factor of TF_ANCHOR_EMA, 0 <= gamma < 1 (the paper
                              uses 0.9); ignored for TF_ANCHOR_MEAN */
    int32_t anchor_inclusive; /* 0 (default): a token is compared with the anchor of the tokens
                              before it (the prose's "previous keys"); 1: with the anchor that
                              already includes the token itself (Algorithm 1 forms its anchor from
                              a K whose last row is the current token) */
} tf_params;

/* Stages of the path, the order of tf_stage_timing_read's output. */
enum { TF_STAGE_SCORE = 0, TF_STAGE_FUSE = 1, TF_STAGE_SELECT = 2, TF_STAGE_COMPACT = 3,
       TF_STAGE_ZERO_ROWS = 4, TF_STAGE_ATTEND = 5, TF_N_STAGES = 6 };

/* Create a context bound to HIP device `device` (made current for the calling thread inside
 * each call).  *out is set only on TF_OK.  tf_destroy(NULL) is a no-op. */
tf_status tf_create(tf_ctx **out, int device);
void tf_destroy(tf_ctx *ctx);

/* Name of a status code; any integer may be passed ("unknown status" for values that are not a
 * tf_status). */
const char *tf_status_string(int status);
/* Text of the last error recorded on `ctx` ("" if none).  Owned by the context. */
const char *tf_last_error(const tf_ctx *ctx);

/* m = seq - floor(r * seq + 1e-6), the number of kept tokens (equals ceil((1 - r) * seq)
 * for ratios with a short decimal expansion).  Returns -1 for seq < 1 or r outside [0, 1). */
int32_t tf_keep_count(int32_t seq, double prune_ratio);

/* Bytes of workspace any of the calls below needs for `p` (0 if p is invalid). */
size_t tf_workspace_bytes(const tf_params *p);

/* Scoring (Algorithm 1 anchor / cosine / mean / var / alpha / s_KV lines; Eq. 2).
 * For each batch row b and position t: per KV head, the cosine of K[b,h,t] with the anchor
 * selected by p->anchor: the mean of K[b,h,0..t-1], or the incremental anchor of Eq. 1 (0 for
 * t = 0; denominator max(|a||x|, 1e-8); clamped to [-1, 1]), the same for V, then the fusion
 * selected by p->fusion.  With TF_FUSE_KEY_ONLY (TF_FUSE_VALUE_ONLY) only K (V) is read, and
 * sim_v (sim_k) is neither computed nor written.
 *   fused  out [batch][seq] float                      required
 *   sim_k  out [batch][n_kv_heads][seq] float          optional (NULL: kept in ws only)
 *   sim_v  out, same shape                             optional */
tf_status tf_score(tf_ctx *ctx, const tf_params *p, const void *K, const void *V, float *fused,
                   float *sim_k, float *sim_v, void *ws, size_t ws_bytes, void *stream);

/* Decision (Algorithm 1 "skip if s_KV > tau", taken at an exact count) and compaction.
 * Per batch row: with m = tf_keep_count(seq, r), tokens 0..min(W, m)-1 are kept, then the
 * m - min(W, m) other tokens with the lowest fused score, equal scores in index order.
 *   fused     in  [batch][seq] float
 *   keep      out [batch][seq] uint8, 1 = kept
 *   kept_idx  out [batch][m] int32, kept positions ascending
 *   tau       out [batch] float: largest score among kept non-forced tokens (+inf when
 *             nothing is filtered, -inf when no non-forced token is kept).  Optional. */
tf_status tf_select(tf_ctx *ctx, const tf_params *p, const float *fused, uint8_t *keep,
                    int32_t *kept_idx, float *tau, void *ws, size_t ws_bytes, void *stream);

/* Causal softmax attention restricted to a kept set (Section 3.2: a skipped token's
 * attention output is zero; the others attend as usual, here to kept tokens only).
 * kept_idx: [batch][m] strictly ascending positions in [0, seq), 1 <= m <= seq; the caller
 * guarantees this, the contents are not checked.  For query
 * head hq the KV head is hq / (n_q_heads / n_kv_heads).  O rows at positions not listed
 * are set to zero.  Arithmetic: fp32 throughout for TF_F32; bf16 MFMA with fp32
 * accumulation and fp32 softmax for TF_BF16. */
tf_status tf_attend(tf_ctx *ctx, const tf_params *p, const void *Q, const void *K,
                    const void *V, const int32_t *kept_idx, int32_t m, void *O, void *ws,
                    size_t ws_bytes, void *stream);

/* Online decision with an adaptive threshold (Algorithm 1, threshold and skip lines; warm-up
 * of Section 3.2; feedback rule of Section 3.3, Eq. 4).  The tokens of a batch row are visited
 * in order; before token t is judged the threshold moves by eta * (P_current - P_target), where
 * P_target = p->prune_ratio and P_current is the fraction of the t tokens seen so far that were
 * skipped; the first p->warmup tokens update the threshold but are never skipped; after that
 * token t is skipped iff fused[t] > tau.  (Eq. 4's sign: the threshold rises when too much has
 * been skipped; Algorithm 1 prints the opposite sign.)  Arithmetic, fixed so that results are
 * reproducible bit for bit: float; P_current = (float)skipped * (1.0f / (float)t) (0 for t = 0);
 * tau = fmaf(eta, P_current - P_target, tau), starting from tau0.  The kept count is whatever the
 * controller produces, one per batch row.
 *   fused     in  [batch][seq] float
 *   keep      out [batch][seq] u8
 *   kept_idx  out [batch][seq] int32: the first count[b] entries of row b are the kept positions
 *                 ascending, the rest is -1
 *   count     out [batch] int32
 *   tau       out [batch] float (optional): the threshold the last token was judged with
 * p->seq up to 2^24 (the count of skipped tokens is carried in a float). */
tf_status tf_select_online(tf_ctx *ctx, const tf_params *p, float eta, float tau0,
                           const float *fused, uint8_t *keep, int32_t *kept_idx, int32_t *count,
                           float *tau, void *ws, size_t ws_bytes, void *stream);

/* tf_attend (Section 3.2: zero attention output for a skipped token, ordinary causal attention
 * for the others) for kept sets whose size differs from row to row, as the online decision of
 * Section 3.3 / Eq. 4 produces them: kept_idx is [batch][seq], row b
 * holds count[b] strictly ascending positions (what follows them is not read); count is a
 * DEVICE array [batch], 0 <= count[b] <= seq.  A row with count 0 gets an all-zero output. */
tf_status tf_attend_ragged(tf_ctx *ctx, const tf_params *p, const void *Q, const void *K,
                           const void *V, const int32_t *kept_idx, const int32_t *count, void *O,
                           void *ws, size_t ws_bytes, void *stream);

/* The whole path with the online decision: tf_score -> tf_select_online -> tf_attend_ragged on
 * one stream, no host round trip.  Outputs as in those calls; tau may be NULL. */
tf_status tf_filtered_attention_online(tf_ctx *ctx, const tf_params *p, float eta, float tau0,
                                       const void *Q, const void *K, const void *V,
                                       uint8_t *keep, int32_t *kept_idx, int32_t *count,
                                       float *fused, float *tau, void *O, void *ws,
                                       size_t ws_bytes, void *stream);

/* The whole layer as Algorithm 1 states it, for every token of every batch row at once: anchor
 * and per-head cosines (Section 3.2), variance-aware fusion (Eq. 2), the skip decision at the
 * target ratio, and attention for the tokens that are not skipped with a zero attention output
 * for those that are (Section 3.2).  tf_score -> tf_select -> tf_attend on one stream, no host
 * round trip.  Outputs as in the three calls above; tau may be NULL. */
tf_status tf_filtered_attention(tf_ctx *ctx, const tf_params *p, const void *Q, const void *K,
                                const void *V, uint8_t *keep, int32_t *kept_idx, float *fused,
                                float *tau, void *O, void *ws, size_t ws_bytes, void *stream);

/* tf_filtered_attention for callers that cannot allocate device memory or bring a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs, kernels and results as tf_filtered_attention, without `ws`: the
 * intermediates (per-head cosines, segment totals) live in a fixed array of
 * TF_STATIC_SCRATCH_BYTES of device memory inside the library (each GPU the library runs on
 * holds it until the process ends).  The call allocates and frees nothing.  A shape for which
 * tf_workspace_bytes(p) exceeds TF_STATIC_SCRATCH_BYTES is rejected with TF_ERR_UNSUPPORTED
 * before anything is enqueued.  All calls on one GPU share the array: two calls that overlap in
 * time on one GPU (different streams, different contexts or threads) race on it; calls that
 * follow each other in one stream do not. */
#define TF_STATIC_SCRATCH_BYTES (16u << 20)
tf_status tf_filtered_attention_static(tf_ctx *ctx, const tf_params *p, const void *Q,
                                       const void *K, const void *V, uint8_t *keep,
                                       int32_t *kept_idx, float *fused, float *tau, void *O,
                                       void *stream);

/* Per-token form of the layer: Algorithm 1 called once per new token of every batch row
 * (anchor of Section 3.2 / Eq. 1, fusion of Eq. 2, warm-up of Section 3.2, threshold rule of
 * Section 3.3 / Eq. 4 exactly as in tf_select_online, zero output for a skipped token).
 * The state lives in caller-owned DEVICE memory described by this host struct:
 *   anchor_k, anchor_v  [batch][n_kv_heads][128] double.  TF_ANCHOR_MEAN: the sums of all keys /
 *                       values seen so far (the mean is formed when a token is scored);
 *                       TF_ANCHOR_EMA: the incremental anchors.  Every token is absorbed, kept or
 *                       skipped.
 *   seen, skipped       [batch] int32: tokens seen / skipped so far
 *   tau                 [batch] float: the threshold
 *   cache_len           [batch] int32: kept tokens in the row's cache
 *   overflow            [batch] int32: set to 1 when a kept token did not fit the cache; that
 *                       token is then handled as a skipped one (zero output, counted as skipped)
 *   k_cache, v_cache    [batch][n_kv_heads][capacity][128] of p->dtype, 16-byte aligned: keys and
 *                       values of the kept tokens in arrival order (a skipped token is neither
 *                       cached nor attended to)
 * p->seq and the strides of `p` are not used by the two calls below (they must still be valid);
 * p->prune_ratio is the target skip ratio, p->warmup the number of tokens never skipped. */
typedef struct {
    double *anchor_k, *anchor_v;
    int32_t *seen, *skipped;
    float *tau;
    int32_t *cache_len, *overflow;
    void *k_cache, *v_cache;
    int32_t capacity; /* rows per (batch, head) in the caches, >= 1 */
    int32_t reserved; /* must be 0 */
} tf_decode_state;

/* Bytes of workspace tf_decode_step needs for `p` (0 if p is invalid). */
size_t tf_decode_workspace_bytes(const tf_params *p);

/* Start a sequence: anchors, counters, cache lengths and overflow flags to zero, tau to tau0. */
tf_status tf_decode_init(tf_ctx *ctx, const tf_params *p, const tf_decode_state *state, float tau0,
                         void *stream);

/* Prompt, then decoding: tf_filtered_attention_online over a prompt of p->seq tokens (same
 * arguments and outputs; the threshold after the last prompt token is written to state->tau),
 * followed by the hand-off that leaves `state` exactly as p->seq calls of tf_decode_step from
 * tf_decode_init(tau0) would have left it (anchors to rounding): anchors over all prompt rows,
 * seen = seq, skipped = seq - count, cache_len = count, overflow = 0, and the kept rows of K and V
 * copied to the caches in order.  state->capacity >= p->seq is required (the prompt may keep
 * every token).  ws as for the batched calls (tf_workspace_bytes). */
tf_status tf_decode_prefill(tf_ctx *ctx, const tf_params *p, float eta, float tau0,
                            const tf_decode_state *state, const void *Q, const void *K,
                            const void *V, uint8_t *keep, int32_t *kept_idx, int32_t *count,
                            float *fused, void *O, void *ws, size_t ws_bytes, void *stream);

/* One new token per batch row.  In this order: the token's key and value are scored against the
 * anchors as they stand; tau <- fmaf(eta, (float)skipped * (1.0f / (float)seen) - target, tau)
 * (P_current = 0 before the first token); the token is skipped iff seen >= p->warmup and
 * fused > tau; the anchors absorb the token; a kept token is appended to the caches and its
 * queries attend over the row's whole cache, itself included.  Run over a sequence from
 * tf_decode_init this equals tf_filtered_attention_online on that sequence (scores to rounding;
 * decisions equal whenever the scores compare equally with the thresholds).
 *   q       in  [batch][n_q_heads][128], k, v  in [batch][n_kv_heads][128], contiguous, p->dtype
 *   o       out [batch][n_q_heads][128]: attention output, all zero for a skipped token
 *   skip    out [batch] u8: 1 = skipped
 *   fused   out [batch] float: the score S_KV the decision was taken on */
tf_status tf_decode_step(tf_ctx *ctx, const tf_params *p, float eta, const tf_decode_state *state,
                         const void *q, const void *k, const void *v, void *o, uint8_t *skip,
                         float *fused, void *ws, size_t ws_bytes, void *stream);

/* Tail-focused layer schedule (Section 3.3, Eq. 3), host side: to meet the global budget
 * p_global in [0, 1], the last ceil(tail_fraction * n_layers) layers (0 < tail_fraction <= 1)
 * are pruned at p_global / tail_fraction (capped at 1: such a layer skips the attention of all
 * its tokens, which tf_filtered_attention_layers accepts), the others at 0.
 * ratios: host array [n_layers]; *n_tail (may be NULL): number of selected layers. */
tf_status tf_tail_schedule(int32_t n_layers, double p_global, double tail_fraction,
                           double *ratios, int32_t *n_tail);

/* Tail-focused multi-layer driver (Section 3.3, Eq. 3: the selected layers run the filter of
 * Algorithm 1 at P_tail, the others are left dense; a skipped token's attention output is zero,
 * Section 3.2): the whole path on n_layers layers of one shape `p`, layer l at pruning ratio
 * ratios[l] (p->prune_ratio is ignored; every ratio in [0, 1], as tf_tail_schedule produces).
 * A layer at ratio 0 does no scoring: all its tokens are kept (keep = 1, kept_idx = 0..seq-1,
 * tau = +inf, fused not written) and it runs plain causal attention.  A layer at ratio 1 (the
 * schedule's cap, e.g. a 50 % budget on the last half of the layers) skips the attention of
 * every token: keep = 0, tau = -inf, O all zero, kept_idx and fused neither read nor written
 * (their pointers may be NULL).  Q, K, V, O, keep,
 * kept_idx, fused, tau: host arrays of n_layers device pointers, each as in
 * tf_filtered_attention (kept_idx[l] holds [batch][tf_keep_count(seq, ratios[l])]); tau may be
 * NULL.  One workspace of tf_workspace_bytes(p) serves all layers in stream order. */
tf_status tf_filtered_attention_layers(tf_ctx *ctx, const tf_params *p, int32_t n_layers,
                                       const double *ratios, const void *const *Q,
                                       const void *const *K, const void *const *V,
                                       uint8_t *const *keep, int32_t *const *kept_idx,
                                       float *const *fused, float *const *tau, void *const *O,
                                       void *ws, size_t ws_bytes, void *stream);

/* Per-stage device timing for measurement.  While enabled, every tf_filtered_attention call
 * brackets its stages with events on the caller's stream (at most 256 calls are recorded
 * between reads).  tf_stage_timing_read waits for those events, writes the summed
 * milliseconds per stage to ms[TF_N_STAGES] and the number of recorded calls to *n_calls,
 * and clears the record.  Enabling costs a few event records per call. */
tf_status tf_stage_timing_enable(tf_ctx *ctx, int on);
tf_status tf_stage_timing_read(tf_ctx *ctx, float *ms, int32_t *n_calls);

/* Measurement probes, not part of the path: what this device reaches on the two resources the
 * path's rooflines are quoted against, to put next to the vendor peaks.  Both enqueue one
 * warm-up and one timed launch on `stream`, wait for them, and return the rate of the timed
 * launch.  `sink` is 4 bytes of device memory (never written in practice).
 * tf_probe_hbm_read: a plain streaming read of `bytes` bytes (a multiple of 16) of device
 *   memory at `src`, 16-byte aligned; *gb_per_s = bytes / time.
 * tf_probe_mfma_bf16: `iters` rounds of four independent v_mfma_f32_32x32x16_bf16 per wave, two
 *   waves per SIMD on every CU; *tflop_per_s = issued flops / time. */
tf_status tf_probe_hbm_read(tf_ctx *ctx, const void *src, size_t bytes, void *sink, void *stream,
                            double *gb_per_s);
tf_status tf_probe_mfma_bf16(tf_ctx *ctx, int32_t iters, void *sink, void *stream,
                             double *tflop_per_s);

#ifdef __cplusplus
}
#endif
#endif /* TOKFILT_H */
