// Host-only calls of the C ABI for a build of csrc/tokfilt_api.hip whose HOST code is compiled
// with AddressSanitizer and UndefinedBehaviorSanitizer (tests/test_host_api_sanitizers.py builds
// and runs it; no GPU is needed or used).  Exit status 0 = every call behaved as documented.
#include "tokfilt.h"
#include <stdio.h>
#include <string.h>
#include <math.h>
int main() {
    int bad = 0;
    for (int n = 1; n < 300; n += 7)
        for (int r = 0; r < 100; r += 3) { int m = tf_keep_count(n, r / 100.0); if (m < 0 || m > n) ++bad; }
    double ratios[40]; int nt = 0;
    if (tf_tail_schedule(40, 0.33, 0.4, ratios, &nt) != TF_OK || nt != 16) ++bad;
    if (tf_tail_schedule(1, 0.9, 0.5, ratios, NULL) != TF_OK || ratios[0] != 1.0) ++bad;
    if (tf_tail_schedule(0, 0.9, 0.5, ratios, NULL) != TF_ERR_INVALID_ARG) ++bad;
    tf_params p; memset(&p, 0, sizeof p);
    p.batch = 2; p.n_q_heads = 8; p.n_kv_heads = 2; p.seq = 300; p.head_dim = 128; p.dtype = TF_BF16;
    long long qs[3] = {8*300*128, 300*128, 128}, ks[3] = {2*300*128, 300*128, 128};
    for (int i = 0; i < 3; ++i) { p.q_stride[i] = qs[i]; p.o_stride[i] = qs[i]; p.kv_stride[i] = ks[i]; }
    p.prune_ratio = 0.5; p.warmup = 1;
    if (tf_workspace_bytes(&p) == 0) ++bad;
    if (tf_decode_workspace_bytes(&p) == 0) ++bad;
    p.head_dim = 64; if (tf_workspace_bytes(&p) != 0) ++bad; p.head_dim = 128;
    p.batch = 70000; if (tf_workspace_bytes(&p) != 0) ++bad; p.batch = 2;
    if (tf_workspace_bytes(NULL) != 0) ++bad;
    for (int s = -1; s < 7; ++s) if (!tf_status_string(s)) ++bad;
    if (strcmp(tf_last_error(NULL), "") != 0) ++bad;
    tf_destroy(NULL);
    tf_ctx* c = NULL;
    tf_status st = tf_create(&c, 0);     // no GPU here: must fail cleanly
    if (st == TF_OK) tf_destroy(c);
    if (tf_create(NULL, 0) != TF_ERR_INVALID_ARG) ++bad;
    // every device entry point refuses a NULL context before touching anything
    if (tf_score(NULL, &p, 0, 0, 0, 0, 0, 0, 0, 0) != TF_ERR_INVALID_ARG) ++bad;
    if (tf_filtered_attention(NULL, &p, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0) != TF_ERR_INVALID_ARG) ++bad;
    if (tf_filtered_attention_static(NULL, &p, 0, 0, 0, 0, 0, 0, 0, 0, 0) != TF_ERR_INVALID_ARG) ++bad;
    printf("host api driver: %d failures\n", bad);
    return bad ? 1 : 0;
}
