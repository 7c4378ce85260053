/*
 * CPU oracle for the Token Filtering hot path.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, double-precision restatement of what the paper defines, used to check the
 * HIP library.  Nothing in the product path may call into this file; it shares no code,
 * header or table with the GPU sources.
 *
 * Paper passages followed (arxiv 2512.07090, "Leveraging KV Similarity for Online Structured
 * Pruning in LLMs"):
 *   - anchor = mean of all previous keys / values, one vector per head:
 *       Algorithm 1 (anchor lines), Section 3.2 paragraph on the anchor key;
 *   - per-head cosine similarity between anchor and current key / value: Algorithm 1,
 *       Section 3.2 (similarity computed per head, then averaged over heads);
 *   - mean and variance over heads, variance-aware fusion: Algorithm 1, Eq. 2;
 *   - skip decision "skip iff S_KV > tau": Algorithm 1 last line, Section 3.3;
 *   - a skipped token's attention output is zero: Section 3.2, paragraph after Algorithm 1;
 *   - attention over the remaining tokens is ordinary causal softmax attention.
 *
 * Readings where the paper is silent or inconsistent (each is also listed in the design
 * document):
 *   - the anchor of token t excludes token t (prose: "previous"); token 0 has a zero anchor;
 *     the other reading (Algorithm 1 forms the anchor from a K that already holds the current
 *     token) is available as the flag `inclusive` of the anchor functions;
 *   - cosine denominator is max(|a| |x|, 1e-8) and the cosine is clamped to [-1, 1];
 *   - the variance is the population variance across heads for one token; 1e-12 is added to
 *     each variance before it is used in alpha;
 *   - fusion mode 0 is alpha exactly as printed in Eq. 2 / Algorithm 1, mode 1 is the
 *     inverse-variance weighting the prose describes, modes 2 / 3 are key-only / value-only;
 *   - the threshold is realised as an exact count: the m = n - floor(r n + 1e-6) tokens with
 *     the lowest score are kept, ties broken towards the lower index, after force-keeping
 *     the first W tokens (warm-up); the decision is taken on the score rounded to float,
 *     the precision the GPU path decides in;
 *   - filtered tokens are neither queries nor keys;
 *   - the per-token form (tfo_decode_step) keeps the anchors over ALL earlier tokens, kept or
 *     skipped (the anchor is the mean of previous keys, not of cached keys), and caches only
 *     kept tokens; token by token it reproduces the batched functions exactly.
 *
 * Parity pins live in tests/test_oracle_pins.py.  Unpinned by the paper (fixed only by the
 * readings above): fusion direction, warm-up length, the two epsilons, the tie-break.
 *
 * Layout everywhere: X[b][h][t][c], c contiguous, float inputs (bf16 inputs are widened
 * exactly by the caller), double arithmetic, double outputs unless stated.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define TFO_EPS_COS 1e-8
#define TFO_EPS_VAR 1e-12

int tfo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Threads the parallel loops over (batch, head) use from now on (for timing on one thread). */
void tfo_set_num_threads(int n)
{
#ifdef _OPENMP
    omp_set_num_threads(n < 1 ? 1 : n);
#else
    (void)n;
#endif
}

/* Incremental anchor (Section 3.2, Eq. 1): Anchor <- gamma * Anchor + (1 - gamma) * x_current,
 * one anchor per (b, h), starting from zero.  inclusive = 0: row t is scored against the anchor
 * as it stands BEFORE row t is folded in (the reading "previous keys" of the exact mean, kept
 * here), so token 0 meets a zero anchor and scores 0 through the guard on the denominator.
 * inclusive = 1: the anchor is updated first and row t is scored against the updated anchor
 * (the order in which Algorithm 1 lists its steps).
 * cosv: [B][H][n].  anchors (optional, may be NULL): [B][H][n][d], the anchor each row met. */
void tfo_anchor_cosine_ema(const float *X, int64_t B, int64_t H, int64_t n, int64_t d,
                           double gamma, int inclusive, double *cosv, double *anchors)
{
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t h = 0; h < H; ++h) {
            double *anchor = (double *)calloc((size_t)d, sizeof(double));
            const float *xbh = X + ((b * H + h) * n) * d;
            for (int64_t t = 0; t < n; ++t) {
                const float *x = xbh + t * d;
                if (inclusive)
                    for (int64_t c = 0; c < d; ++c)
                        anchor[c] = gamma * anchor[c] + (1.0 - gamma) * (double)x[c];
                if (anchors)
                    memcpy(anchors + (((b * H + h) * n) + t) * d, anchor,
                           (size_t)d * sizeof(double));
                double dot = 0.0, na = 0.0, nx = 0.0;
                for (int64_t c = 0; c < d; ++c) {
                    double xc = (double)x[c];
                    dot += anchor[c] * xc;
                    na += anchor[c] * anchor[c];
                    nx += xc * xc;
                }
                double den = sqrt(na) * sqrt(nx);
                if (den < TFO_EPS_COS)
                    den = TFO_EPS_COS;
                double cs = dot / den;
                if (cs > 1.0)
                    cs = 1.0;
                if (cs < -1.0)
                    cs = -1.0;
                cosv[(b * H + h) * n + t] = cs;
                if (!inclusive)
                    for (int64_t c = 0; c < d; ++c)
                        anchor[c] = gamma * anchor[c] + (1.0 - gamma) * (double)x[c];
            }
            free(anchor);
        }
    }
}

/* Anchor (Algorithm 1, anchor lines; Section 3.2): for each (b, h, t) the mean of rows
 * 0..t-1 of X[b][h] (inclusive = 1: of rows 0..t, the current row included, which is what
 * Algorithm 1's mean over a K that ends with the current token says literally), and the cosine
 * similarity of that mean with row t.
 * cosv: [B][H][n].  anchors (optional, may be NULL): [B][H][n][d], the means themselves. */
void tfo_anchor_cosine(const float *X, int64_t B, int64_t H, int64_t n, int64_t d,
                       int inclusive, double *cosv, double *anchors)
{
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t h = 0; h < H; ++h) {
            double *sum = (double *)calloc((size_t)d, sizeof(double));
            double *anchor = (double *)calloc((size_t)d, sizeof(double));
            const float *xbh = X + ((b * H + h) * n) * d;
            for (int64_t t = 0; t < n; ++t) {
                const float *x = xbh + t * d;
                if (inclusive)
                    for (int64_t c = 0; c < d; ++c)
                        sum[c] += (double)x[c];
                int64_t rows = inclusive ? t + 1 : t;
                for (int64_t c = 0; c < d; ++c)
                    anchor[c] = (rows == 0) ? 0.0 : sum[c] / (double)rows;
                if (anchors)
                    memcpy(anchors + (((b * H + h) * n) + t) * d, anchor,
                           (size_t)d * sizeof(double));
                double dot = 0.0, na = 0.0, nx = 0.0;
                for (int64_t c = 0; c < d; ++c) {
                    double xc = (double)x[c];
                    dot += anchor[c] * xc;
                    na += anchor[c] * anchor[c];
                    nx += xc * xc;
                }
                double den = sqrt(na) * sqrt(nx);
                if (den < TFO_EPS_COS)
                    den = TFO_EPS_COS;
                double cs = dot / den;
                if (cs > 1.0)
                    cs = 1.0;
                if (cs < -1.0)
                    cs = -1.0;
                cosv[(b * H + h) * n + t] = cs;
                if (!inclusive)
                    for (int64_t c = 0; c < d; ++c)
                        sum[c] += (double)x[c];
            }
            free(sum);
            free(anchor);
        }
    }
}

/* Head statistics and fusion (Algorithm 1 mean/var lines; Eq. 2).
 * cK, cV: [B][H][n] per-head cosines.  mode: 0 Eq. 2 as printed, 1 inverse-variance as in
 * the prose, 2 key only, 3 value only.
 * S: [B][n].  stats (optional): [B][n][5] = s_k, s_v, var_k, var_v, alpha. */
void tfo_fuse(const double *cK, const double *cV, int64_t B, int64_t H, int64_t n, int mode,
              double *S, double *stats)
{
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t t = 0; t < n; ++t) {
            double sk = 0.0, sv = 0.0;
            for (int64_t h = 0; h < H; ++h) {
                sk += cK[(b * H + h) * n + t];
                sv += cV[(b * H + h) * n + t];
            }
            sk /= (double)H;
            sv /= (double)H;
            double vk = 0.0, vv = 0.0;
            for (int64_t h = 0; h < H; ++h) {
                double dk = cK[(b * H + h) * n + t] - sk;
                double dv = cV[(b * H + h) * n + t] - sv;
                vk += dk * dk;
                vv += dv * dv;
            }
            vk /= (double)H;
            vv /= (double)H;
            double ek = vk + TFO_EPS_VAR, ev = vv + TFO_EPS_VAR;
            double alpha;
            if (mode == 0)
                alpha = (1.0 / ev) / (1.0 / ek + 1.0 / ev); /* Eq. 2 exactly as printed */
            else if (mode == 1)
                alpha = (1.0 / ek) / (1.0 / ek + 1.0 / ev); /* weight on the steadier side */
            else if (mode == 2)
                alpha = 1.0;
            else
                alpha = 0.0;
            S[b * n + t] = alpha * sk + (1.0 - alpha) * sv;
            if (stats) {
                double *st = stats + (b * n + t) * 5;
                st[0] = sk;
                st[1] = sv;
                st[2] = vk;
                st[3] = vv;
                st[4] = alpha;
            }
        }
    }
}

/* Tail-focused layer schedule (Section 3.3, Eq. 3): to meet a global budget p_global the last
 * fraction y of the layers is pruned at p_tail = p_global / y (not above 1) and the other layers
 * are not pruned at all.  Reading: "the last y fraction" of L layers is the last ceil(y * L - 1e-9)
 * of them.  ratios: [n_layers], front layers 0.  Returns the number of selected layers, or -1
 * for arguments outside n_layers >= 1, 0 <= p_global <= 1, 0 < y <= 1. */
int64_t tfo_tail_schedule(int64_t n_layers, double p_global, double y, double *ratios)
{
    if (n_layers < 1 || !(p_global >= 0.0 && p_global <= 1.0) || !(y > 0.0 && y <= 1.0))
        return -1;
    int64_t n_tail = (int64_t)ceil(y * (double)n_layers - 1e-9);
    if (n_tail < 1)
        n_tail = 1;
    double p_tail = p_global / y;
    if (p_tail > 1.0)
        p_tail = 1.0;
    for (int64_t l = 0; l < n_layers; ++l)
        ratios[l] = (l >= n_layers - n_tail) ? p_tail : 0.0;
    return n_tail;
}

/* Number of kept tokens for pruning ratio r over n tokens. */
int64_t tfo_keep_count(int64_t n, double r)
{
    return n - (int64_t)floor(r * (double)n + 1e-6);
}

typedef struct {
    float s;
    int32_t idx;
} tfo_pair;

static int tfo_pair_cmp(const void *a, const void *b)
{
    const tfo_pair *pa = (const tfo_pair *)a, *pb = (const tfo_pair *)b;
    if (pa->s < pb->s)
        return -1;
    if (pa->s > pb->s)
        return 1;
    return (pa->idx > pb->idx) - (pa->idx < pb->idx);
}

/* Decision (Algorithm 1 last line, with the exact-count reading): per batch row keep the
 * first min(W, m) tokens, then the m - min(W, m) remaining tokens with the lowest score
 * (ties: lower index first).  S32: [B][n] scores already rounded to float.
 * keep: [B][n] 0/1.  kept_idx: [B][m] ascending positions.  tau: [B] = largest score among
 * kept non-forced tokens; +inf if nothing is filtered, -inf if no non-forced token is kept. */
void tfo_select(const float *S32, int64_t B, int64_t n, int64_t m, int64_t W, uint8_t *keep,
                int32_t *kept_idx, float *tau)
{
    for (int64_t b = 0; b < B; ++b) {
        const float *s = S32 + b * n;
        uint8_t *kp = keep + b * n;
        int64_t forced = W < m ? W : m;
        if (forced < 0)
            forced = 0;
        memset(kp, 0, (size_t)n);
        for (int64_t t = 0; t < forced; ++t)
            kp[t] = 1;
        int64_t rest = n - forced, want = m - forced;
        tfo_pair *p = (tfo_pair *)malloc((size_t)(rest > 0 ? rest : 1) * sizeof(tfo_pair));
        for (int64_t t = forced; t < n; ++t) {
            p[t - forced].s = s[t];
            p[t - forced].idx = (int32_t)t;
        }
        qsort(p, (size_t)rest, sizeof(tfo_pair), tfo_pair_cmp);
        float tb;
        if (m >= n)
            tb = INFINITY;
        else if (want <= 0)
            tb = -INFINITY;
        else
            tb = p[want - 1].s;
        for (int64_t i = 0; i < want; ++i)
            kp[p[i].idx] = 1;
        free(p);
        tau[b] = tb;
        int64_t c = 0;
        for (int64_t t = 0; t < n; ++t)
            if (kp[t])
                kept_idx[b * m + c++] = (int32_t)t;
    }
}

/* Online decision with an adaptive threshold (Algorithm 1, threshold and skip lines; warm-up of
 * Section 3.2; feedback rule of Section 3.3, Eq. 4).  Tokens of a row are visited in order.
 * Before token t is judged the threshold moves by eta * (P_current - P_target), where P_current
 * is the fraction of the t tokens seen so far that were skipped (0 for t = 0); the threshold is
 * updated during the first W tokens too, but those are never skipped; after that token t is
 * skipped iff S_t > tau.
 * Readings.  (1) Sign: Eq. 4 (tau rises when too much has been skipped, negative feedback) is
 * followed; Algorithm 1 prints eta * (target - current), which would push the ratio away from the
 * target.  (2) Arithmetic, fixed so that an implementation can agree bit for bit: everything in
 * float; P_current = (float)skipped * (1.0f / (float)t); tau = fmaf(eta, P_current - target, tau).
 * S32: [B][n].  keep: [B][n] 0/1.  kept_idx: [B][n], the first count[b] entries of row b are the
 * kept positions ascending, the rest is -1.  count: [B].  tau_out: [B], the threshold after the
 * last token.  tau_trace (may be NULL): [B][n], the threshold each token was judged with. */
void tfo_select_online(const float *S32, int64_t B, int64_t n, int64_t W, float target, float eta,
                       float tau0, uint8_t *keep, int32_t *kept_idx, int32_t *count,
                       float *tau_out, float *tau_trace)
{
    for (int64_t b = 0; b < B; ++b) {
        const float *s = S32 + b * n;
        float tau = tau0;
        int64_t skipped = 0, kept = 0;
        for (int64_t t = 0; t < n; ++t) {
            float inv_t = (t == 0) ? 0.0f : 1.0f / (float)t;
            float p_current = (float)skipped * inv_t;
            float diff = p_current - target;
            tau = fmaf(eta, diff, tau);
            if (tau_trace)
                tau_trace[b * n + t] = tau;
            int skip = (t >= W) && (s[t] > tau);
            keep[b * n + t] = (uint8_t)!skip;
            if (skip)
                ++skipped;
            else
                kept_idx[b * n + kept++] = (int32_t)t;
        }
        for (int64_t i = kept; i < n; ++i)
            kept_idx[b * n + i] = -1;
        count[b] = (int32_t)kept;
        tau_out[b] = tau;
    }
}

/* One output row of causal softmax attention restricted to the kept tokens: query at kept
 * rank i of (b, hq) attends kept ranks 0..i of kv head hq / (Hq / Hkv).  out: [d]. */
static void tfo_attend_one(const float *Q, const float *K, const float *V, int64_t Hq,
                           int64_t Hkv, int64_t n, int64_t d, const int32_t *idx, int64_t i,
                           int64_t b, int64_t hq, double scale, double *logits, double *out)
{
    int64_t hk = hq / (Hq / Hkv);
    const float *q = Q + (((b * Hq + hq) * n) + idx[i]) * d;
    const float *Kbh = K + ((b * Hkv + hk) * n) * d;
    const float *Vbh = V + ((b * Hkv + hk) * n) * d;
    double mx = -INFINITY;
    for (int64_t j = 0; j <= i; ++j) {
        const float *k = Kbh + (int64_t)idx[j] * d;
        double acc = 0.0;
        for (int64_t c = 0; c < d; ++c)
            acc += (double)q[c] * (double)k[c];
        logits[j] = acc * scale;
        if (logits[j] > mx)
            mx = logits[j];
    }
    double z = 0.0;
    for (int64_t j = 0; j <= i; ++j) {
        logits[j] = exp(logits[j] - mx);
        z += logits[j];
    }
    for (int64_t c = 0; c < d; ++c)
        out[c] = 0.0;
    for (int64_t j = 0; j <= i; ++j) {
        const float *v = Vbh + (int64_t)idx[j] * d;
        double wj = logits[j] / z;
        for (int64_t c = 0; c < d; ++c)
            out[c] += wj * (double)v[c];
    }
}

/* Attention over kept tokens for the whole layer (Section 3.2: zero output for skipped
 * tokens; standard causal attention otherwise).  Q: [B][Hq][n][d]; K, V: [B][Hkv][n][d];
 * kept_idx: [B][m]; O: [B][Hq][n][d], rows of filtered positions are exactly zero. */
void tfo_attend(const float *Q, const float *K, const float *V, int64_t B, int64_t Hq,
                int64_t Hkv, int64_t n, int64_t d, const int32_t *kept_idx, int64_t m,
                double scale, double *O)
{
    memset(O, 0, (size_t)(B * Hq * n * d) * sizeof(double));
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t hq = 0; hq < Hq; ++hq) {
            double *logits = (double *)malloc((size_t)(m > 0 ? m : 1) * sizeof(double));
            const int32_t *idx = kept_idx + b * m;
            for (int64_t i = 0; i < m; ++i)
                tfo_attend_one(Q, K, V, Hq, Hkv, n, d, idx, i, b, hq, scale, logits,
                               O + (((b * Hq + hq) * n) + idx[i]) * d);
            free(logits);
        }
    }
}

/* The same definition for a list of sampled output rows: rows[r] = (b, hq, kept rank i);
 * out: [R][d].  Used where the full layer is too large to recompute on the CPU. */
void tfo_attend_rows(const float *Q, const float *K, const float *V, int64_t B, int64_t Hq,
                     int64_t Hkv, int64_t n, int64_t d, const int32_t *kept_idx, int64_t m,
                     double scale, const int32_t *rows, int64_t R, double *out)
{
    (void)B;
#pragma omp parallel for schedule(dynamic)
    for (int64_t r = 0; r < R; ++r) {
        int64_t b = rows[3 * r], hq = rows[3 * r + 1], i = rows[3 * r + 2];
        double *logits = (double *)malloc((size_t)(i + 1) * sizeof(double));
        tfo_attend_one(Q, K, V, Hq, Hkv, n, d, kept_idx + b * m, i, b, hq, scale, logits,
                       out + r * d);
        free(logits);
    }
}

/* One decoding step of the Token Filtering layer for every batch row (Algorithm 1 as a per-token
 * call; anchor of Section 3.2 / Eq. 1; fusion of Eq. 2; warm-up of Section 3.2; threshold rule of
 * Section 3.3, Eq. 4; zero attention output for a skipped token, Section 3.2).
 * State carried between calls (all owned by the caller, one entry per batch row unless stated):
 *   anchor_k, anchor_v [B][Hkv][d] double: anchor kind 0: sums of all rows seen so far (the mean
 *       is formed when a row is scored); kind 1: the incremental anchors of Eq. 1;
 *   seen, skipped: tokens seen / skipped so far;  tau: the threshold (float);
 *   cache_len: rows held in the cache;  k_cache, v_cache [B][Hkv][capacity][d]: keys / values of
 *       the kept tokens in arrival order.
 * Steps, in this order: the new key and value are scored against the anchors as they stand (they
 * include every earlier token, kept or not, and not the current one; with inclusive = 1 against
 * the anchors as they will stand once the current token is absorbed);
 * the threshold moves exactly as in tfo_select_online (float arithmetic); the token is skipped
 * iff seen >= W and S > tau (S rounded to float); the anchors absorb the token; a kept token is
 * appended to the cache and attends over the whole cache, itself included (a skipped token is
 * neither cached nor attended to, and its output is zero).
 * decide_on (may be NULL): [B] scores to take the decision on in place of this function's own
 * (for comparing an implementation whose scores differ in the last bits).
 * o: [B][Hq][d] double.  skip: [B] 0/1.  fused: [B] double.
 * Returns 0, or -1 if a kept token does not fit its row's cache (nothing is changed then). */
int tfo_decode_step(const float *q, const float *k, const float *v, int64_t B, int64_t Hq,
                    int64_t Hkv, int64_t d, int anchor_kind, double gamma, int inclusive,
                    int fusion, int64_t W,
                    float target, float eta, double scale, const float *decide_on,
                    double *anchor_k, double *anchor_v, int32_t *seen, int32_t *skipped,
                    float *tau, int32_t *cache_len, float *k_cache, float *v_cache,
                    int64_t capacity, double *o, uint8_t *skip, double *fused)
{
    double *ck = (double *)malloc((size_t)(2 * B * Hkv) * sizeof(double));
    double *cv = ck + B * Hkv;
    /* scores against the anchors as they stand */
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t h = 0; h < Hkv; ++h) {
            for (int which = 0; which < 2; ++which) {
                const float *x = (which ? v : k) + (b * Hkv + h) * d;
                const double *a = (which ? anchor_v : anchor_k) + (b * Hkv + h) * d;
                double dot = 0.0, na = 0.0, nx = 0.0;
                for (int64_t c = 0; c < d; ++c) {
                    double ac = a[c];
                    if (anchor_kind == 0) {
                        if (inclusive)
                            ac = (ac + (double)x[c]) / (double)(seen[b] + 1);
                        else
                            ac = seen[b] > 0 ? ac / (double)seen[b] : 0.0;
                    } else if (inclusive) {
                        ac = gamma * ac + (1.0 - gamma) * (double)x[c];
                    }
                    dot += ac * (double)x[c];
                    na += ac * ac;
                    nx += (double)x[c] * (double)x[c];
                }
                double den = sqrt(na) * sqrt(nx);
                if (den < TFO_EPS_COS)
                    den = TFO_EPS_COS;
                double cs = dot / den;
                cs = cs > 1.0 ? 1.0 : (cs < -1.0 ? -1.0 : cs);
                (which ? cv : ck)[b * Hkv + h] = cs;
            }
        }
    }
    tfo_fuse(ck, cv, B, Hkv, 1, fusion, fused, NULL);
    free(ck);
    /* decisions first, so that a full cache is found before any state changes */
    float *new_tau = (float *)malloc((size_t)B * sizeof(float));
    for (int64_t b = 0; b < B; ++b) {
        float inv_t = seen[b] == 0 ? 0.0f : 1.0f / (float)seen[b];
        float p_current = (float)skipped[b] * inv_t;
        float diff = p_current - target;
        new_tau[b] = fmaf(eta, diff, tau[b]);
        float s = decide_on ? decide_on[b] : (float)fused[b];
        skip[b] = (uint8_t)((seen[b] >= W) && (s > new_tau[b]));
        if (!skip[b] && cache_len[b] >= capacity) {
            free(new_tau);
            return -1;
        }
    }
    for (int64_t b = 0; b < B; ++b) {
        tau[b] = new_tau[b];
        for (int64_t h = 0; h < Hkv; ++h) {
            const float *xk = k + (b * Hkv + h) * d, *xv = v + (b * Hkv + h) * d;
            double *ak = anchor_k + (b * Hkv + h) * d, *av = anchor_v + (b * Hkv + h) * d;
            for (int64_t c = 0; c < d; ++c) {
                if (anchor_kind == 0) {
                    ak[c] += (double)xk[c];
                    av[c] += (double)xv[c];
                } else {
                    ak[c] = gamma * ak[c] + (1.0 - gamma) * (double)xk[c];
                    av[c] = gamma * av[c] + (1.0 - gamma) * (double)xv[c];
                }
            }
            if (!skip[b]) {
                memcpy(k_cache + ((b * Hkv + h) * capacity + cache_len[b]) * d, xk,
                       (size_t)d * sizeof(float));
                memcpy(v_cache + ((b * Hkv + h) * capacity + cache_len[b]) * d, xv,
                       (size_t)d * sizeof(float));
            }
        }
        seen[b] += 1;
        if (skip[b])
            skipped[b] += 1;
        else
            cache_len[b] += 1;
    }
    free(new_tau);
    /* attention of the kept tokens over their row's cache */
    for (int64_t b = 0; b < B; ++b) {
        for (int64_t hq = 0; hq < Hq; ++hq) {
            double *out = o + (b * Hq + hq) * d;
            for (int64_t c = 0; c < d; ++c)
                out[c] = 0.0;
            if (skip[b])
                continue;
            int64_t hk = hq / (Hq / Hkv), len = cache_len[b];
            const float *qr = q + (b * Hq + hq) * d;
            const float *Kc = k_cache + (b * Hkv + hk) * capacity * d;
            const float *Vc = v_cache + (b * Hkv + hk) * capacity * d;
            double *logit = (double *)malloc((size_t)len * sizeof(double));
            double mx = -INFINITY, z = 0.0;
            for (int64_t j = 0; j < len; ++j) {
                double acc = 0.0;
                for (int64_t c = 0; c < d; ++c)
                    acc += (double)qr[c] * (double)Kc[j * d + c];
                logit[j] = acc * scale;
                if (logit[j] > mx)
                    mx = logit[j];
            }
            for (int64_t j = 0; j < len; ++j) {
                logit[j] = exp(logit[j] - mx);
                z += logit[j];
            }
            for (int64_t j = 0; j < len; ++j)
                for (int64_t c = 0; c < d; ++c)
                    out[c] += logit[j] / z * (double)Vc[j * d + c];
            free(logit);
        }
    }
    return 0;
}
