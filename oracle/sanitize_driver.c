/*
 * Drives every entry point of the CPU oracle once on small, odd-sized inputs.  TEST
 * INFRASTRUCTURE ONLY: built together with tokfilt_oracle.c under -fsanitize=address,undefined
 * by tests/test_oracle_sanitizers.py, which expects exit status 0 and no sanitizer report.
 * Every buffer is allocated at exactly the size the oracle's comments state, so a read or
 * write past an end is caught.  Prints one checksum line.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void tfo_set_num_threads(int n);
void tfo_anchor_cosine_ema(const float *X, int64_t B, int64_t H, int64_t n, int64_t d, double gamma,
                           int inclusive, double *cosv, double *anchors);
void tfo_anchor_cosine(const float *X, int64_t B, int64_t H, int64_t n, int64_t d, int inclusive,
                       double *cosv, double *anchors);
void tfo_fuse(const double *cK, const double *cV, int64_t B, int64_t H, int64_t n, int mode, double *S,
              double *stats);
int64_t tfo_tail_schedule(int64_t n_layers, double p_global, double y, double *ratios);
int64_t tfo_keep_count(int64_t n, double r);
void tfo_select(const float *S32, int64_t B, int64_t n, int64_t m, int64_t W, uint8_t *keep,
                int32_t *kept_idx, float *tau);
void tfo_select_online(const float *S32, int64_t B, int64_t n, int64_t W, float target, float eta,
                       float tau0, uint8_t *keep, int32_t *kept_idx, int32_t *count, float *tau_out,
                       float *tau_trace);
void tfo_attend(const float *Q, const float *K, const float *V, int64_t B, int64_t Hq, int64_t Hkv,
                int64_t n, int64_t d, const int32_t *kept_idx, int64_t m, double scale, double *O);
void tfo_attend_rows(const float *Q, const float *K, const float *V, int64_t B, int64_t Hq,
                     int64_t Hkv, int64_t n, int64_t d, const int32_t *kept_idx, int64_t m,
                     double scale, const int32_t *rows, int64_t R, double *out);
int tfo_decode_step(const float *q, const float *k, const float *v, int64_t B, int64_t Hq, int64_t Hkv,
                    int64_t d, int anchor_kind, double gamma, int inclusive, int fusion, int64_t W,
                    float target, float eta, double scale, const float *decide_on, double *anchor_k,
                    double *anchor_v, int32_t *seen, int32_t *skipped, float *tau, int32_t *cache_len,
                    float *k_cache, float *v_cache, int64_t capacity, double *o, uint8_t *skip,
                    double *fused);

static uint32_t rng_state = 12345u;
static float rnd(void)
{
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)((rng_state >> 8) & 0xffff) / 32768.0f - 1.0f;
}
static float *rand_floats(size_t count)
{
    float *p = (float *)malloc(count * sizeof(float));
    for (size_t i = 0; i < count; ++i)
        p[i] = rnd();
    return p;
}

int main(void)
{
    const int64_t B = 2, Hq = 6, Hkv = 3, n = 37, d = 16;
    double check = 0.0;
    tfo_set_num_threads(3);
    float *Q = rand_floats((size_t)(B * Hq * n * d));
    float *K = rand_floats((size_t)(B * Hkv * n * d));
    float *V = rand_floats((size_t)(B * Hkv * n * d));
    double *ck = (double *)malloc((size_t)(B * Hkv * n) * sizeof(double));
    double *cv = (double *)malloc((size_t)(B * Hkv * n) * sizeof(double));
    double *anch = (double *)malloc((size_t)(B * Hkv * n * d) * sizeof(double));
    double *S = (double *)malloc((size_t)(B * n) * sizeof(double));
    double *stats = (double *)malloc((size_t)(B * n * 5) * sizeof(double));
    float *S32 = (float *)malloc((size_t)(B * n) * sizeof(float));
    for (int inclusive = 0; inclusive < 2; ++inclusive) {
        tfo_anchor_cosine(K, B, Hkv, n, d, inclusive, ck, anch);
        tfo_anchor_cosine(V, B, Hkv, n, d, inclusive, cv, NULL);
        tfo_anchor_cosine_ema(K, B, Hkv, n, d, 0.9, inclusive, ck, anch);
        tfo_anchor_cosine_ema(V, B, Hkv, n, d, 0.0, inclusive, cv, NULL);
        for (int mode = 0; mode < 4; ++mode) {
            tfo_fuse(ck, cv, B, Hkv, n, mode, S, mode ? NULL : stats);
            check += S[B * n - 1];
        }
    }
    tfo_anchor_cosine(K, B, Hkv, n, d, 0, ck, NULL);
    tfo_anchor_cosine(V, B, Hkv, n, d, 0, cv, NULL);
    tfo_fuse(ck, cv, B, Hkv, n, 0, S, NULL);
    for (int64_t i = 0; i < B * n; ++i)
        S32[i] = (float)S[i];
    S32[5] = S32[6] = S32[7];                           /* ties */

    const double ratios[] = {0.0, 0.3, 0.5, 0.97, 1.0};
    const int64_t warmups[] = {0, 1, 5, 100};
    for (size_t ri = 0; ri < sizeof(ratios) / sizeof(ratios[0]); ++ri) {
        for (size_t wi = 0; wi < sizeof(warmups) / sizeof(warmups[0]); ++wi) {
            int64_t m = tfo_keep_count(n, ratios[ri]);
            uint8_t *keep = (uint8_t *)malloc((size_t)(B * n));
            int32_t *idx = (int32_t *)malloc((size_t)(B * (m > 0 ? m : 1)) * sizeof(int32_t));
            float *tau = (float *)malloc((size_t)B * sizeof(float));
            tfo_select(S32, B, n, m, warmups[wi], keep, idx, tau);
            if (wi == 1) {
                double *O = (double *)malloc((size_t)(B * Hq * n * d) * sizeof(double));
                tfo_attend(Q, K, V, B, Hq, Hkv, n, d, idx, m, 0.25, O);
                check += O[(B * Hq * n * d) - 1] + O[0];
                if (m > 0) {
                    int32_t rows[6] = {0, 0, 0, (int32_t)(B - 1), (int32_t)(Hq - 1), (int32_t)(m - 1)};
                    double *out = (double *)malloc((size_t)(2 * d) * sizeof(double));
                    tfo_attend_rows(Q, K, V, B, Hq, Hkv, n, d, idx, m, 0.25, rows, 2, out);
                    check += out[2 * d - 1];
                    free(out);
                }
                free(O);
            }
            free(keep);
            free(idx);
            free(tau);
        }
    }
    {
        uint8_t *keep = (uint8_t *)malloc((size_t)(B * n));
        int32_t *idx = (int32_t *)malloc((size_t)(B * n) * sizeof(int32_t));
        int32_t *count = (int32_t *)malloc((size_t)B * sizeof(int32_t));
        float *tau = (float *)malloc((size_t)B * sizeof(float));
        float *trace = (float *)malloc((size_t)(B * n) * sizeof(float));
        tfo_select_online(S32, B, n, 4, 0.5f, 0.05f, 0.2f, keep, idx, count, tau, trace);
        tfo_select_online(S32, B, n, 0, 0.5f, 0.0f, -1.0f, keep, idx, count, tau, NULL);
        check += count[0] + tau[B - 1];
        free(keep); free(idx); free(count); free(tau); free(trace);
    }
    {
        double r[7];
        check += (double)tfo_tail_schedule(7, 0.9, 0.5, r) + r[6];
        check += (double)tfo_tail_schedule(1, 0.2, 1.0, r);
        check += (double)tfo_tail_schedule(0, 0.2, 1.0, r);
    }
    for (int kind = 0; kind < 2; ++kind) {
        const int64_t cap = 9;                           /* smaller than n: the cache fills up */
        double *ak = (double *)calloc((size_t)(B * Hkv * d), sizeof(double));
        double *av = (double *)calloc((size_t)(B * Hkv * d), sizeof(double));
        int32_t *seen = (int32_t *)calloc((size_t)B, sizeof(int32_t));
        int32_t *skipped = (int32_t *)calloc((size_t)B, sizeof(int32_t));
        int32_t *clen = (int32_t *)calloc((size_t)B, sizeof(int32_t));
        float *tau = (float *)malloc((size_t)B * sizeof(float));
        float *kc = (float *)malloc((size_t)(B * Hkv * cap * d) * sizeof(float));
        float *vc = (float *)malloc((size_t)(B * Hkv * cap * d) * sizeof(float));
        double *o = (double *)malloc((size_t)(B * Hq * d) * sizeof(double));
        double *fused = (double *)malloc((size_t)B * sizeof(double));
        uint8_t *skip = (uint8_t *)malloc((size_t)B);
        float *q1 = (float *)malloc((size_t)(B * Hq * d) * sizeof(float));
        float *k1 = (float *)malloc((size_t)(B * Hkv * d) * sizeof(float));
        float *v1 = (float *)malloc((size_t)(B * Hkv * d) * sizeof(float));
        for (int64_t b = 0; b < B; ++b)
            tau[b] = 0.3f;
        int full = 0;
        for (int64_t t = 0; t < n && !full; ++t) {
            for (int64_t b = 0; b < B; ++b) {
                for (int64_t h = 0; h < Hq; ++h)
                    memcpy(q1 + (b * Hq + h) * d, Q + (((b * Hq + h) * n) + t) * d, (size_t)d * sizeof(float));
                for (int64_t h = 0; h < Hkv; ++h) {
                    memcpy(k1 + (b * Hkv + h) * d, K + (((b * Hkv + h) * n) + t) * d, (size_t)d * sizeof(float));
                    memcpy(v1 + (b * Hkv + h) * d, V + (((b * Hkv + h) * n) + t) * d, (size_t)d * sizeof(float));
                }
            }
            int rc = tfo_decode_step(q1, k1, v1, B, Hq, Hkv, d, kind, 0.9, kind, kind, 2, 0.5f, 0.05f, 0.25,
                                     NULL, ak, av, seen, skipped, tau, clen, kc, vc, cap, o, skip, fused);
            if (rc != 0)
                full = 1;                                /* a kept token did not fit: state untouched */
            else
                check += o[B * Hq * d - 1] + fused[0];
        }
        check += (double)seen[0] + (double)clen[B - 1];
        free(ak); free(av); free(seen); free(skipped); free(clen); free(tau); free(kc); free(vc);
        free(o); free(fused); free(skip); free(q1); free(k1); free(v1);
    }
    free(Q); free(K); free(V); free(ck); free(cv); free(anch); free(S); free(stats); free(S32);
    if (!isfinite(check)) {
        fprintf(stderr, "checksum is not finite\n");
        return 2;
    }
    printf("oracle sanitizer driver: checksum %.6f\n", check);
    return 0;
}
