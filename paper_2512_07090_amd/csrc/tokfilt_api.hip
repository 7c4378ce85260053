// C ABI of the token-filter library: argument checking, workspace carving and the order in
// which the kernels are enqueued.  All arithmetic of the method lives in the kernels.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <new>

#include "../../include/tokfilt.h"
#include "tf_kernels.h"

// Scratch of tf_filtered_attention_static: a fixed array in device memory, one copy per GPU the
// library is loaded on, held until the process ends.  In host code this name is only a handle
// for hipGetSymbolAddress; the address kernels and copies use is the one kept in the context.
static __device__ __align__(256) unsigned char scratch[TF_STATIC_SCRATCH_BYTES];

struct tf_ctx {
    int device;
    int n_cu;   // compute units of the device
    int n_xcd;  // accelerator dies (each has its own L2)
    void* static_scratch;  // device address of `scratch` on this context's GPU
    char err[256];
    int timing_on;
    int timing_calls;
    hipEvent_t ev[256][TF_N_STAGES + 1];
    bool ev_ready;
};

namespace {

constexpr int kMaxTimedCalls = 256;
constexpr int kMaxKvHeads = 128;  // LDS staging of the fusion kernel
constexpr int kMaxOnlineSeq = 1 << 24;  // the online decision's float counter of skipped tokens is exact up to here

tf_status fail(tf_ctx* c, tf_status s, const char* fmt, ...) __attribute__((format(printf, 3, 4)));
tf_status fail(tf_ctx* c, tf_status s, const char* fmt, ...)
{
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return s;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Workspace {
    size_t sim_k, sim_v, seg_tot, keep_tmp, total;  // byte offsets
};

// Pure shape validation, usable without a context.
tf_status check_shape(const tf_params* p, const char** why)
{
    *why = "";
    if (!p) { *why = "params is NULL"; return TF_ERR_INVALID_ARG; }
    if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->seq < 1) {
        *why = "batch, head counts and seq must be >= 1"; return TF_ERR_INVALID_ARG;
    }
    if (p->n_q_heads % p->n_kv_heads != 0) {
        *why = "n_q_heads must be a multiple of n_kv_heads"; return TF_ERR_INVALID_ARG;
    }
    if (p->dtype != TF_F32 && p->dtype != TF_BF16) { *why = "unknown dtype"; return TF_ERR_INVALID_ARG; }
    if (p->fusion < TF_FUSE_EQ2 || p->fusion > TF_FUSE_VALUE_ONLY) {
        *why = "unknown fusion mode"; return TF_ERR_INVALID_ARG;
    }
    if (!(p->prune_ratio >= 0.0 && p->prune_ratio < 1.0)) {
        *why = "prune_ratio must be in [0, 1)"; return TF_ERR_INVALID_ARG;
    }
    if (p->warmup < 0) { *why = "warmup must be >= 0"; return TF_ERR_INVALID_ARG; }
    if (p->anchor_inclusive != 0 && p->anchor_inclusive != 1) { *why = "anchor_inclusive must be 0 or 1"; return TF_ERR_INVALID_ARG; }
    if (p->anchor != TF_ANCHOR_MEAN && p->anchor != TF_ANCHOR_EMA) { *why = "unknown anchor"; return TF_ERR_INVALID_ARG; }
    if (p->anchor == TF_ANCHOR_EMA && !(p->ema_gamma >= 0.f && p->ema_gamma < 1.f)) {
        *why = "ema_gamma must be in [0, 1)"; return TF_ERR_INVALID_ARG;
    }
    if (!(p->softmax_scale >= 0.f) || isinf(p->softmax_scale)) {
        *why = "softmax_scale must be finite and >= 0"; return TF_ERR_INVALID_ARG;
    }
    const int64_t* st[3] = {p->q_stride, p->kv_stride, p->o_stride};
    for (int a = 0; a < 3; ++a)
        for (int i = 0; i < 3; ++i)
            if (st[a][i] < 0 || st[a][i] % 8 != 0 || (i == 2 && st[a][i] < p->head_dim)) {
                *why = "strides must be non-negative multiples of 8 elements, position stride >= head_dim";
                return TF_ERR_INVALID_ARG;
            }
    if (p->head_dim != tf::kHeadDim) { *why = "only head_dim 128 is supported"; return TF_ERR_UNSUPPORTED; }
    if (p->n_kv_heads > kMaxKvHeads) { *why = "more than 128 KV heads is not supported"; return TF_ERR_UNSUPPORTED; }
    if ((int64_t)p->batch * p->seq > (int64_t)1 << 30) { *why = "batch * seq too large"; return TF_ERR_UNSUPPORTED; }
    if (p->dtype == TF_BF16 && (p->seq > (1 << 24) || p->kv_stride[2] * 2 >= (1 << 24) ||
                                (int64_t)p->seq * p->kv_stride[2] * 2 >= ((int64_t)1 << 32))) {
        *why = "a (batch, head) slice of K / V must span less than 4 GiB (bf16 attention addresses rows by 32-bit offsets)";
        return TF_ERR_UNSUPPORTED;
    }
    // batch rows and query heads index the second and third grid dimension of some launches
    if (p->batch > 65535 || p->n_q_heads > 65535) {
        *why = "batch and n_q_heads above 65535 are not supported"; return TF_ERR_UNSUPPORTED;
    }
    return TF_OK;
}

// which tensors the scoring kernel has to walk: 0 = both, 1 = K only, 2 = V only
int score_tensors(const tf_params* p)
{
    return p->fusion == TF_FUSE_KEY_ONLY ? 1 : (p->fusion == TF_FUSE_VALUE_ONLY ? 2 : 0);
}

// anchor kind and the inclusive flag as the scoring launcher takes them
int anchor_bits(const tf_params* p) { return p->anchor | (p->anchor_inclusive << 1); }

tf::Dims make_dims(const tf_params* p, int m)
{
    tf::Dims d;
    d.B = p->batch; d.Hq = p->n_q_heads; d.Hkv = p->n_kv_heads; d.n = p->seq; d.m = m;
    for (int i = 0; i < 3; ++i) { d.qs[i] = p->q_stride[i]; d.kvs[i] = p->kv_stride[i]; d.os[i] = p->o_stride[i]; }
    return d;
}

Workspace carve(const tf_params* p)
{
    const tf::Dims d = make_dims(p, 0);
    Workspace w;
    const size_t sims = align256((size_t)p->batch * p->n_kv_heads * p->seq * sizeof(float));
    size_t off = 0;
    w.sim_k = off; off += sims;
    w.sim_v = off; off += sims;
    w.seg_tot = off; off += align256(tf::score_scratch_floats(d) * sizeof(float));
    w.keep_tmp = off; off += align256((size_t)p->batch * p->seq);
    w.total = off;
    return w;
}

bool misaligned(const void* p) { return ((uintptr_t)p & 15) != 0; }

tf_status enter(tf_ctx* ctx, const tf_params* p, void* ws, size_t ws_bytes, Workspace* w)
{
    if (!ctx) return TF_ERR_INVALID_ARG;
    const char* why;
    const tf_status s = check_shape(p, &why);
    if (s != TF_OK) return fail(ctx, s, "%s", why);
    *w = carve(p);
    if (!ws) return fail(ctx, TF_ERR_INVALID_ARG, "workspace pointer is NULL");
    if (misaligned(ws)) return fail(ctx, TF_ERR_INVALID_ARG, "workspace must be 16-byte aligned");
    if (ws_bytes < w->total)
        return fail(ctx, TF_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, w->total);
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipSetDevice(%d) failed", ctx->device);
    return TF_OK;
}

tf_status dev(tf_ctx* ctx, hipError_t e, const char* what)
{
    if (e == hipSuccess) return TF_OK;
    return fail(ctx, TF_ERR_DEVICE, "%s: %s", what, hipGetErrorString(e));
}

void mark(tf_ctx* ctx, int slot, int stage, hipStream_t s)
{
    if (slot >= 0) (void)hipEventRecord(ctx->ev[slot][stage], s);
}

// counts (may be null): per-row kept counts on the device; kept_idx rows are then p->seq apart
// and d.m is the bound p->seq
tf_status run_attend(tf_ctx* ctx, const tf_params* p, const tf::Dims& d, const void* Q,
                     const void* K, const void* V, const int32_t* kept_idx,
                     const uint8_t* keep, void* O, hipStream_t s, int slot,
                     const int32_t* counts = nullptr)
{
    const float scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
    if (p->dtype == TF_F32) {
        tf_status st = dev(ctx, tf::launch_zero_filtered(d, p->dtype, keep, O, s), "zero-fill launch");
        if (st != TF_OK) return st;
        mark(ctx, slot, TF_STAGE_ATTEND, s);
        return dev(ctx, tf::launch_attend_f32(d, scale, (const float*)Q, (const float*)K, (const float*)V,
                                              kept_idx, (float*)O, counts, p->seq, s), "fp32 attention launch");
    }
    // the bf16 kernel writes the zero rows itself
    mark(ctx, slot, TF_STAGE_ATTEND, s);
    return dev(ctx, tf::launch_attend_bf16(d, scale, Q, K, V, kept_idx, O, ctx->n_cu, ctx->n_xcd, counts, p->seq, s),
               "bf16 attention launch");
}

// validation shared by the decode calls; fills everything of `a` the state and params determine
tf_status decode_args(tf_ctx* ctx, const tf_params* p, const tf_decode_state* st, tf::DecodeArgs* a)
{
    const char* why;
    const tf_status s = check_shape(p, &why);
    if (s != TF_OK) return fail(ctx, s, "%s", why);
    if (!st) return fail(ctx, TF_ERR_INVALID_ARG, "state is NULL");
    if (!st->anchor_k || !st->anchor_v || !st->seen || !st->skipped || !st->tau || !st->cache_len ||
        !st->overflow || !st->k_cache || !st->v_cache)
        return fail(ctx, TF_ERR_INVALID_ARG, "a pointer of the decode state is NULL");
    if (st->capacity < 1 || st->reserved != 0)
        return fail(ctx, TF_ERR_INVALID_ARG, "decode state: capacity must be >= 1 and reserved 0");
    if (misaligned(st->k_cache) || misaligned(st->v_cache) || misaligned(st->anchor_k) || misaligned(st->anchor_v))
        return fail(ctx, TF_ERR_INVALID_ARG, "caches and anchors must be 16-byte aligned");
    if ((int64_t)p->batch * p->n_kv_heads * (int64_t)st->capacity > ((int64_t)1 << 40) / tf::kHeadDim)
        return fail(ctx, TF_ERR_UNSUPPORTED, "cache too large");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipSetDevice(%d) failed", ctx->device);
    a->B = p->batch; a->Hq = p->n_q_heads; a->Hkv = p->n_kv_heads; a->capacity = st->capacity;
    a->anchor_k = st->anchor_k; a->anchor_v = st->anchor_v;
    a->seen = st->seen; a->skipped = st->skipped; a->cache_len = st->cache_len; a->overflow = st->overflow;
    a->tau = st->tau; a->k_cache = st->k_cache; a->v_cache = st->v_cache;
    a->ema = p->anchor == TF_ANCHOR_EMA; a->inclusive = p->anchor_inclusive; a->fusion = p->fusion; a->warmup = p->warmup;
    a->gamma = (double)p->ema_gamma;
    a->target = (float)p->prune_ratio; a->eta = 0.f;
    a->scale = p->softmax_scale > 0.f ? p->softmax_scale : 1.0f / sqrtf((float)p->head_dim);
    a->skip = nullptr; a->fused = nullptr; a->part = nullptr; a->n_split = 1;
    return TF_OK;
}

}  // namespace

namespace {

// score -> fuse -> select + compact -> attend for one layer (arguments already validated)
tf_status run_path(tf_ctx* ctx, const tf_params* p, const Workspace& w, const void* Q,
                   const void* K, const void* V, uint8_t* keep, int32_t* kept_idx, float* fused,
                   float* tau, void* O, void* ws, hipStream_t s)
{
    const tf::Dims d = make_dims(p, tf_keep_count(p->seq, p->prune_ratio));
    char* base = (char*)ws;
    float* sk = (float*)(base + w.sim_k);
    float* sv = (float*)(base + w.sim_v);

    int slot = -1;
    if (ctx->timing_on && ctx->timing_calls < kMaxTimedCalls) slot = ctx->timing_calls++;

    mark(ctx, slot, 0, s);
    tf_status st = dev(ctx, tf::launch_score(d, p->dtype, K, V, sk, sv, (float*)(base + w.seg_tot),
                                             score_tensors(p), anchor_bits(p), p->ema_gamma, s), "score launch");
    if (st != TF_OK) return st;
    mark(ctx, slot, 1, s);
    st = dev(ctx, tf::launch_fuse(d, p->fusion, sk, sv, fused, s), "fuse launch");
    if (st != TF_OK) return st;
    mark(ctx, slot, 2, s);
    st = dev(ctx, tf::launch_select_compact(d, p->warmup, fused, keep, kept_idx, tau, s),
             "select launch");
    if (st != TF_OK) return st;
    mark(ctx, slot, 3, s);  // compaction is part of the decision kernel
    mark(ctx, slot, 4, s);
    st = run_attend(ctx, p, d, Q, K, V, kept_idx, keep, O, s, slot);
    if (st != TF_OK) return st;
    mark(ctx, slot, TF_N_STAGES, s);
    return TF_OK;
}

// one warm-up and one timed launch of `launch`, milliseconds of the timed one
template <class F>
tf_status time_probe(tf_ctx* ctx, hipStream_t s, F launch, float* ms)
{
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipEventCreate failed");
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(ctx, TF_ERR_DEVICE, "hipEventCreate failed");
    }
    hipError_t e = launch();
    if (e == hipSuccess) e = hipEventRecord(e0, s);
    if (e == hipSuccess) e = launch();
    if (e == hipSuccess) e = hipEventRecord(e1, s);
    if (e == hipSuccess) e = hipEventSynchronize(e1);
    if (e == hipSuccess) e = hipEventElapsedTime(ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return dev(ctx, e, "probe");
}

}  // namespace

extern "C" {

tf_status tf_create(tf_ctx** out, int device)
{
    if (!out) return TF_ERR_INVALID_ARG;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return TF_ERR_DEVICE;
    tf_ctx* c = new (std::nothrow) tf_ctx;
    if (!c) return TF_ERR_DEVICE;
    memset(c, 0, sizeof(*c));
    c->device = device;
    if (hipDeviceGetAttribute(&c->n_cu, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || c->n_cu < 1) {
        delete c;
        return TF_ERR_DEVICE;
    }
    if (hipDeviceGetAttribute(&c->n_xcd, hipDeviceAttributeNumberOfXccs, device) != hipSuccess || c->n_xcd < 1)
        c->n_xcd = 1;  // unknown: one run of groups; only cache locality depends on it
    // every GPU holds its own copy of the static scratch array at its own address: ask for it
    // with this context's device current
    if (hipSetDevice(device) != hipSuccess ||
        hipGetSymbolAddress(&c->static_scratch, HIP_SYMBOL(scratch)) != hipSuccess || !c->static_scratch) {
        delete c;
        return TF_ERR_DEVICE;
    }
    *out = c;
    return TF_OK;
}

void tf_destroy(tf_ctx* ctx)
{
    if (!ctx) return;
    if (ctx->ev_ready) {
        (void)hipSetDevice(ctx->device);
        for (int i = 0; i < kMaxTimedCalls; ++i)
            for (int j = 0; j <= TF_N_STAGES; ++j) (void)hipEventDestroy(ctx->ev[i][j]);
    }
    delete ctx;
}

const char* tf_status_string(int status)
{
    switch (status) {
        case TF_OK: return "ok";
        case TF_ERR_INVALID_ARG: return "invalid argument";
        case TF_ERR_UNSUPPORTED: return "unsupported configuration";
        case TF_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case TF_ERR_DEVICE: return "device error";
    }
    return "unknown status";
}

const char* tf_last_error(const tf_ctx* ctx) { return ctx ? ctx->err : ""; }

int32_t tf_keep_count(int32_t seq, double prune_ratio)
{
    if (seq < 1 || !(prune_ratio >= 0.0 && prune_ratio < 1.0)) return -1;
    return seq - (int32_t)floor(prune_ratio * (double)seq + 1e-6);
}

size_t tf_workspace_bytes(const tf_params* p)
{
    const char* why;
    if (check_shape(p, &why) != TF_OK) return 0;
    return carve(p).total;
}

tf_status tf_score(tf_ctx* ctx, const tf_params* p, const void* K, const void* V, float* fused,
                   float* sim_k, float* sim_v, void* ws, size_t ws_bytes, void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    if (!K || !V || !fused) return fail(ctx, TF_ERR_INVALID_ARG, "K, V and fused must not be NULL");
    if (misaligned(K) || misaligned(V)) return fail(ctx, TF_ERR_INVALID_ARG, "K and V must be 16-byte aligned");
    const tf::Dims d = make_dims(p, tf_keep_count(p->seq, p->prune_ratio));
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)ws;
    float* sk = sim_k ? sim_k : (float*)(base + w.sim_k);
    float* sv = sim_v ? sim_v : (float*)(base + w.sim_v);
    st = dev(ctx, tf::launch_score(d, p->dtype, K, V, sk, sv, (float*)(base + w.seg_tot), score_tensors(p), anchor_bits(p), p->ema_gamma, s), "score launch");
    if (st != TF_OK) return st;
    return dev(ctx, tf::launch_fuse(d, p->fusion, sk, sv, fused, s), "fuse launch");
}

tf_status tf_select(tf_ctx* ctx, const tf_params* p, const float* fused, uint8_t* keep,
                    int32_t* kept_idx, float* tau, void* ws, size_t ws_bytes, void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    if (!fused || !keep || !kept_idx) return fail(ctx, TF_ERR_INVALID_ARG, "fused, keep and kept_idx must not be NULL");
    const tf::Dims d = make_dims(p, tf_keep_count(p->seq, p->prune_ratio));
    hipStream_t s = (hipStream_t)stream;
    return dev(ctx, tf::launch_select_compact(d, p->warmup, fused, keep, kept_idx, tau, s),
               "select launch");
}

tf_status tf_attend(tf_ctx* ctx, const tf_params* p, const void* Q, const void* K, const void* V,
                    const int32_t* kept_idx, int32_t m, void* O, void* ws, size_t ws_bytes,
                    void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    if (!Q || !K || !V || !O || !kept_idx) return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V, O and kept_idx must not be NULL");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V and O must be 16-byte aligned");
    if (m < 1 || m > p->seq) return fail(ctx, TF_ERR_INVALID_ARG, "m must be in [1, seq]");
    const tf::Dims d = make_dims(p, m);
    hipStream_t s = (hipStream_t)stream;
    uint8_t* keep = (uint8_t*)((char*)ws + w.keep_tmp);
    if (p->dtype == TF_F32) {  // the fp32 path zero-fills from a mask
        st = dev(ctx, tf::launch_mask_from_idx(d, kept_idx, keep, nullptr, 0, s), "mask launch");
        if (st != TF_OK) return st;
    }
    return run_attend(ctx, p, d, Q, K, V, kept_idx, keep, O, s, -1);
}

tf_status tf_select_online(tf_ctx* ctx, const tf_params* p, float eta, float tau0,
                           const float* fused, uint8_t* keep, int32_t* kept_idx, int32_t* count,
                           float* tau, void* ws, size_t ws_bytes, void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    if (!fused || !keep || !kept_idx || !count)
        return fail(ctx, TF_ERR_INVALID_ARG, "fused, keep, kept_idx and count must not be NULL");
    if (!(eta >= 0.f) || isinf(eta) || isnan(tau0) || isinf(tau0))
        return fail(ctx, TF_ERR_INVALID_ARG, "eta must be finite and >= 0, tau0 finite");
    if (p->seq > kMaxOnlineSeq)
        return fail(ctx, TF_ERR_UNSUPPORTED, "the online decision counts skipped tokens in a float: seq above 2^24 is not supported");
    const tf::Dims d = make_dims(p, p->seq);
    return dev(ctx, tf::launch_select_online(d, p->warmup, (float)p->prune_ratio, eta, tau0, fused, keep,
                                             kept_idx, count, tau, (hipStream_t)stream),
               "online decision launch");
}

tf_status tf_attend_ragged(tf_ctx* ctx, const tf_params* p, const void* Q, const void* K,
                           const void* V, const int32_t* kept_idx, const int32_t* count, void* O,
                           void* ws, size_t ws_bytes, void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    if (!Q || !K || !V || !O || !kept_idx || !count)
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V, O, kept_idx and count must not be NULL");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V and O must be 16-byte aligned");
    const tf::Dims d = make_dims(p, p->seq);
    hipStream_t s = (hipStream_t)stream;
    uint8_t* keep = (uint8_t*)((char*)ws + w.keep_tmp);
    if (p->dtype == TF_F32) {  // the fp32 path zero-fills from a mask
        st = dev(ctx, tf::launch_mask_from_idx(d, kept_idx, keep, count, p->seq, s), "mask launch");
        if (st != TF_OK) return st;
    }
    return run_attend(ctx, p, d, Q, K, V, kept_idx, keep, O, s, -1, count);
}

tf_status tf_filtered_attention_online(tf_ctx* ctx, const tf_params* p, float eta, float tau0,
                                       const void* Q, const void* K, const void* V, uint8_t* keep,
                                       int32_t* kept_idx, int32_t* count, float* fused, float* tau,
                                       void* O, void* ws, size_t ws_bytes, void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    if (!Q || !K || !V || !O || !keep || !kept_idx || !count || !fused)
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V, O, keep, kept_idx, count and fused must not be NULL");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V and O must be 16-byte aligned");
    if (!(eta >= 0.f) || isinf(eta) || isnan(tau0) || isinf(tau0))
        return fail(ctx, TF_ERR_INVALID_ARG, "eta must be finite and >= 0, tau0 finite");
    if (p->seq > kMaxOnlineSeq)
        return fail(ctx, TF_ERR_UNSUPPORTED, "the online decision counts skipped tokens in a float: seq above 2^24 is not supported");
    const tf::Dims d = make_dims(p, p->seq);
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)ws;
    float* sk = (float*)(base + w.sim_k);
    float* sv = (float*)(base + w.sim_v);
    st = dev(ctx, tf::launch_score(d, p->dtype, K, V, sk, sv, (float*)(base + w.seg_tot),
                                   score_tensors(p), anchor_bits(p), p->ema_gamma, s), "score launch");
    if (st != TF_OK) return st;
    st = dev(ctx, tf::launch_fuse(d, p->fusion, sk, sv, fused, s), "fuse launch");
    if (st != TF_OK) return st;
    st = dev(ctx, tf::launch_select_online(d, p->warmup, (float)p->prune_ratio, eta, tau0, fused, keep,
                                           kept_idx, count, tau, s), "online decision launch");
    if (st != TF_OK) return st;
    return run_attend(ctx, p, d, Q, K, V, kept_idx, keep, O, s, -1, count);
}

size_t tf_decode_workspace_bytes(const tf_params* p)
{
    const char* why;
    if (check_shape(p, &why) != TF_OK) return 0;
    return align256((size_t)p->batch * p->n_q_heads * tf::kDecodeMaxSplit * tf::kDecodePartFloats * sizeof(float));
}

tf_status tf_decode_init(tf_ctx* ctx, const tf_params* p, const tf_decode_state* state, float tau0,
                         void* stream)
{
    if (!ctx) return TF_ERR_INVALID_ARG;
    tf::DecodeArgs a;
    tf_status st = decode_args(ctx, p, state, &a);
    if (st != TF_OK) return st;
    if (isnan(tau0) || isinf(tau0)) return fail(ctx, TF_ERR_INVALID_ARG, "tau0 must be finite");
    return dev(ctx, tf::launch_decode_init(a, tau0, (hipStream_t)stream), "decode init launch");
}

tf_status tf_decode_prefill(tf_ctx* ctx, const tf_params* p, float eta, float tau0,
                            const tf_decode_state* state, const void* Q, const void* K,
                            const void* V, uint8_t* keep, int32_t* kept_idx, int32_t* count,
                            float* fused, void* O, void* ws, size_t ws_bytes, void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    tf::DecodeArgs a;
    st = decode_args(ctx, p, state, &a);
    if (st != TF_OK) return st;
    if (state->capacity < p->seq)
        return fail(ctx, TF_ERR_INVALID_ARG, "the caches hold %d rows, the prompt may keep %d", state->capacity, p->seq);
    if ((int64_t)p->batch * p->n_kv_heads > 65535)
        return fail(ctx, TF_ERR_UNSUPPORTED, "batch * n_kv_heads above 65535 is not supported by the hand-off");
    if (!Q || !K || !V || !O || !keep || !kept_idx || !count || !fused)
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V, O, keep, kept_idx, count and fused must not be NULL");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V and O must be 16-byte aligned");
    if (!(eta >= 0.f) || isinf(eta) || isnan(tau0) || isinf(tau0))
        return fail(ctx, TF_ERR_INVALID_ARG, "eta must be finite and >= 0, tau0 finite");
    if (p->seq > kMaxOnlineSeq)
        return fail(ctx, TF_ERR_UNSUPPORTED, "the online decision counts skipped tokens in a float: seq above 2^24 is not supported");
    const tf::Dims d = make_dims(p, p->seq);
    hipStream_t s = (hipStream_t)stream;
    char* base = (char*)ws;
    float* sk = (float*)(base + w.sim_k);
    float* sv = (float*)(base + w.sim_v);
    st = dev(ctx, tf::launch_score(d, p->dtype, K, V, sk, sv, (float*)(base + w.seg_tot),
                                   score_tensors(p), anchor_bits(p), p->ema_gamma, s), "score launch");
    if (st != TF_OK) return st;
    st = dev(ctx, tf::launch_fuse(d, p->fusion, sk, sv, fused, s), "fuse launch");
    if (st != TF_OK) return st;
    // the threshold after the last prompt token goes straight into the state
    st = dev(ctx, tf::launch_select_online(d, p->warmup, (float)p->prune_ratio, eta, tau0, fused, keep,
                                           kept_idx, count, state->tau, s), "online decision launch");
    if (st != TF_OK) return st;
    st = run_attend(ctx, p, d, Q, K, V, kept_idx, keep, O, s, -1, count);
    if (st != TF_OK) return st;
    return dev(ctx, tf::launch_decode_seed(a, p->dtype, K, V, kept_idx, count, p->seq, d.kvs, s),
               "decode state hand-off launch");
}

tf_status tf_decode_step(tf_ctx* ctx, const tf_params* p, float eta, const tf_decode_state* state,
                         const void* q, const void* k, const void* v, void* o, uint8_t* skip,
                         float* fused, void* ws, size_t ws_bytes, void* stream)
{
    if (!ctx) return TF_ERR_INVALID_ARG;
    tf::DecodeArgs a;
    tf_status st = decode_args(ctx, p, state, &a);
    if (st != TF_OK) return st;
    if (!q || !k || !v || !o || !skip || !fused)
        return fail(ctx, TF_ERR_INVALID_ARG, "q, k, v, o, skip and fused must not be NULL");
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(o))
        return fail(ctx, TF_ERR_INVALID_ARG, "q, k, v and o must be 16-byte aligned");
    if (!(eta >= 0.f) || isinf(eta)) return fail(ctx, TF_ERR_INVALID_ARG, "eta must be finite and >= 0");
    if (!ws || misaligned(ws)) return fail(ctx, TF_ERR_INVALID_ARG, "workspace must be a 16-byte aligned pointer");
    const size_t need = tf_decode_workspace_bytes(p);
    if (ws_bytes < need)
        return fail(ctx, TF_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", ws_bytes, need);
    a.eta = eta;
    a.skip = skip;
    a.fused = fused;
    a.part = (float*)ws;
    // enough workgroups for about four per compute unit, each slice at least one pass of keys
    const int group = p->n_q_heads / p->n_kv_heads;
    const int heads_per_wg = (group == 2 || group == 4 || group == 8) ? group : 1;
    const int rows = p->batch * (p->n_q_heads / heads_per_wg);
    int n_split = (4 * ctx->n_cu + rows - 1) / rows;
    n_split = n_split < 1 ? 1 : (n_split > tf::kDecodeMaxSplit ? tf::kDecodeMaxSplit : n_split);
    const int by_len = (state->capacity + 63) / 64;
    a.n_split = n_split > by_len ? by_len : n_split;
    return dev(ctx, tf::launch_decode_step(a, p->dtype, q, k, v, o, (hipStream_t)stream), "decode step launch");
}

tf_status tf_filtered_attention(tf_ctx* ctx, const tf_params* p, const void* Q, const void* K,
                                const void* V, uint8_t* keep, int32_t* kept_idx, float* fused,
                                float* tau, void* O, void* ws, size_t ws_bytes, void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    if (!Q || !K || !V || !O || !keep || !kept_idx || !fused)
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V, O, keep, kept_idx and fused must not be NULL");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V and O must be 16-byte aligned");
    return run_path(ctx, p, w, Q, K, V, keep, kept_idx, fused, tau, O, ws, (hipStream_t)stream);
}

tf_status tf_filtered_attention_static(tf_ctx* ctx, const tf_params* p, const void* Q,
                                       const void* K, const void* V, uint8_t* keep,
                                       int32_t* kept_idx, float* fused, float* tau, void* O,
                                       void* stream)
{
    if (!ctx) return TF_ERR_INVALID_ARG;
    const char* why;
    const tf_status s = check_shape(p, &why);
    if (s != TF_OK) return fail(ctx, s, "%s", why);
    const Workspace w = carve(p);
    if (w.total > (size_t)TF_STATIC_SCRATCH_BYTES)
        return fail(ctx, TF_ERR_UNSUPPORTED,
                    "this shape needs %zu bytes of scratch, the static scratch holds %zu: use "
                    "tf_filtered_attention with a workspace", w.total, (size_t)TF_STATIC_SCRATCH_BYTES);
    if (!Q || !K || !V || !O || !keep || !kept_idx || !fused)
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V, O, keep, kept_idx and fused must not be NULL");
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O))
        return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V and O must be 16-byte aligned");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipSetDevice(%d) failed", ctx->device);
    // nothing in the scratch has to start at zero: every kernel of the path writes what it reads
    return run_path(ctx, p, w, Q, K, V, keep, kept_idx, fused, tau, O, ctx->static_scratch, (hipStream_t)stream);
}

tf_status tf_tail_schedule(int32_t n_layers, double p_global, double tail_fraction,
                           double* ratios, int32_t* n_tail)
{
    if (n_layers < 1 || !ratios || !(p_global >= 0.0 && p_global <= 1.0) ||
        !(tail_fraction > 0.0 && tail_fraction <= 1.0))
        return TF_ERR_INVALID_ARG;
    int32_t nt = (int32_t)ceil(tail_fraction * (double)n_layers - 1e-9);
    if (nt < 1) nt = 1;
    const double p_tail = fmin(p_global / tail_fraction, 1.0);
    for (int32_t l = 0; l < n_layers; ++l) ratios[l] = l >= n_layers - nt ? p_tail : 0.0;
    if (n_tail) *n_tail = nt;
    return TF_OK;
}

tf_status tf_filtered_attention_layers(tf_ctx* ctx, const tf_params* p, int32_t n_layers,
                                       const double* ratios, const void* const* Q,
                                       const void* const* K, const void* const* V,
                                       uint8_t* const* keep, int32_t* const* kept_idx,
                                       float* const* fused, float* const* tau, void* const* O,
                                       void* ws, size_t ws_bytes, void* stream)
{
    Workspace w;
    tf_status st = enter(ctx, p, ws, ws_bytes, &w);
    if (st != TF_OK) return st;
    if (n_layers < 1 || !ratios || !Q || !K || !V || !O || !keep || !kept_idx || !fused)
        return fail(ctx, TF_ERR_INVALID_ARG, "n_layers >= 1 and the ratio and pointer arrays are required");
    // everything is checked before the first launch
    for (int32_t l = 0; l < n_layers; ++l) {
        if (!(ratios[l] >= 0.0 && ratios[l] <= 1.0))
            return fail(ctx, TF_ERR_INVALID_ARG, "ratio of layer %d must be in [0, 1]", l);
        const bool scored = ratios[l] > 0.0 && ratios[l] < 1.0;
        if (!Q[l] || !K[l] || !V[l] || !O[l] || !keep[l] || (ratios[l] < 1.0 && !kept_idx[l]) || (scored && !fused[l]))
            return fail(ctx, TF_ERR_INVALID_ARG, "a pointer of layer %d is NULL", l);
        if (misaligned(Q[l]) || misaligned(K[l]) || misaligned(V[l]) || misaligned(O[l]))
            return fail(ctx, TF_ERR_INVALID_ARG, "Q, K, V and O of layer %d must be 16-byte aligned", l);
    }
    hipStream_t s = (hipStream_t)stream;
    for (int32_t l = 0; l < n_layers; ++l) {
        tf_params pl = *p;
        pl.prune_ratio = ratios[l];
        float* tau_l = tau ? tau[l] : nullptr;
        if (ratios[l] >= 1.0) {
            // the schedule's cap (P_global / Y reaching 1): the attention of every token of this
            // layer is skipped, so no scoring, no kept token, an all-zero output
            pl.prune_ratio = 0.0;
            const tf::Dims d = make_dims(&pl, 0);
            st = dev(ctx, tf::launch_keep_none(d, keep[l], tau_l, s), "keep-none launch");
            if (st == TF_OK) st = dev(ctx, tf::launch_zero_filtered(d, p->dtype, keep[l], O[l], s), "zero-fill launch");
        } else if (tf_keep_count(p->seq, ratios[l]) == p->seq) {
            // nothing to filter: no scoring, every token kept, plain causal attention
            const tf::Dims d = make_dims(&pl, p->seq);
            st = dev(ctx, tf::launch_keep_all(d, keep[l], kept_idx[l], tau_l, s), "keep-all launch");
            if (st == TF_OK) st = run_attend(ctx, &pl, d, Q[l], K[l], V[l], kept_idx[l], keep[l], O[l], s, -1);
        } else {
            st = run_path(ctx, &pl, w, Q[l], K[l], V[l], keep[l], kept_idx[l], fused[l], tau_l, O[l], ws, s);
        }
        if (st != TF_OK) return st;
    }
    return TF_OK;
}

tf_status tf_stage_timing_enable(tf_ctx* ctx, int on)
{
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipSetDevice failed");
    if (on && !ctx->ev_ready) {
        for (int i = 0; i < kMaxTimedCalls; ++i)
            for (int j = 0; j <= TF_N_STAGES; ++j)
                if (hipEventCreate(&ctx->ev[i][j]) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipEventCreate failed");
        ctx->ev_ready = true;
    }
    ctx->timing_on = on ? 1 : 0;
    ctx->timing_calls = 0;
    return TF_OK;
}

tf_status tf_stage_timing_read(tf_ctx* ctx, float* ms, int32_t* n_calls)
{
    if (!ctx || !ms || !n_calls) return TF_ERR_INVALID_ARG;
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipSetDevice failed");
    for (int j = 0; j < TF_N_STAGES; ++j) ms[j] = 0.f;
    for (int i = 0; i < ctx->timing_calls; ++i) {
        if (hipEventSynchronize(ctx->ev[i][TF_N_STAGES]) != hipSuccess)
            return fail(ctx, TF_ERR_DEVICE, "hipEventSynchronize failed");
        for (int j = 0; j < TF_N_STAGES; ++j) {
            float t = 0.f;
            if (hipEventElapsedTime(&t, ctx->ev[i][j], ctx->ev[i][j + 1]) != hipSuccess)
                return fail(ctx, TF_ERR_DEVICE, "hipEventElapsedTime failed");
            ms[j] += t;
        }
    }
    *n_calls = ctx->timing_calls;
    ctx->timing_calls = 0;
    return TF_OK;
}

tf_status tf_probe_hbm_read(tf_ctx* ctx, const void* src, size_t bytes, void* sink, void* stream,
                            double* gb_per_s)
{
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (!src || !sink || !gb_per_s || bytes < 16 || bytes % 16 != 0 || misaligned(src))
        return fail(ctx, TF_ERR_INVALID_ARG, "src (16-byte aligned), sink, gb_per_s and a positive multiple of 16 bytes are required");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipSetDevice(%d) failed", ctx->device);
    hipStream_t s = (hipStream_t)stream;
    float ms = 0.f;
    const tf_status st = time_probe(ctx, s, [&] { return tf::launch_probe_stream_read(src, bytes, sink, ctx->n_cu, s); }, &ms);
    if (st != TF_OK) return st;
    *gb_per_s = (double)bytes / ((double)ms * 1e-3) / 1e9;
    return TF_OK;
}

tf_status tf_probe_mfma_bf16(tf_ctx* ctx, int32_t iters, void* sink, void* stream, double* tflop_per_s)
{
    if (!ctx) return TF_ERR_INVALID_ARG;
    if (!sink || !tflop_per_s || iters < 1) return fail(ctx, TF_ERR_INVALID_ARG, "sink, tflop_per_s and iters >= 1 are required");
    if (hipSetDevice(ctx->device) != hipSuccess) return fail(ctx, TF_ERR_DEVICE, "hipSetDevice(%d) failed", ctx->device);
    hipStream_t s = (hipStream_t)stream;
    float ms = 0.f;
    const tf_status st = time_probe(ctx, s, [&] { return tf::launch_probe_mfma(iters, sink, ctx->n_cu, s); }, &ms);
    if (st != TF_OK) return st;
    const double flops = (double)ctx->n_cu * 8.0 * (double)iters * 4.0 * (2.0 * 32 * 32 * 16);
    *tflop_per_s = flops / ((double)ms * 1e-3) / 1e12;
    return TF_OK;
}

}  // extern "C"
