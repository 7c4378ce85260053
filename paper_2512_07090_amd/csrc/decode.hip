// Per-token form of the layer (Algorithm 1 called once per new token): score the new key and
// value against the caller-held anchors, move the threshold, decide, absorb the token into the
// anchors, append a kept token to the cache of kept keys / values and attend over that cache.
// Three launches per step: decode_score_kernel (one workgroup per batch row), the split
// attention over the cache, and the merge of the splits.
#include <algorithm>

#include "tf_kernels.h"

namespace tf {

namespace {

constexpr double kEpsCos = 1e-8;
constexpr double kEpsVar = 1e-12;
constexpr float kLowest = -1e30f;  // "no key yet": finite, so differences of two of them are 0
constexpr int kPartStride = kDecodePartFloats;  // partial result: 128 numerators, running max, sum

// eight consecutive elements of a row as floats
__device__ __forceinline__ void load8(const uint16_t* p, float* x)
{
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    const unsigned w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        x[2 * i] = __uint_as_float(w[i] << 16);
        x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}
__device__ __forceinline__ void load8(const float* p, float* x)
{
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    x[0] = a.x; x[1] = a.y; x[2] = a.z; x[3] = a.w;
    x[4] = b.x; x[5] = b.y; x[6] = b.z; x[7] = b.w;
}
__device__ __forceinline__ void copy8(uint16_t* dst, const uint16_t* src)
{
    *reinterpret_cast<uint4*>(dst) = *reinterpret_cast<const uint4*>(src);
}
__device__ __forceinline__ void copy8(float* dst, const float* src)
{
    reinterpret_cast<float4*>(dst)[0] = reinterpret_cast<const float4*>(src)[0];
    reinterpret_cast<float4*>(dst)[1] = reinterpret_cast<const float4*>(src)[1];
}
__device__ __forceinline__ void store_out(uint16_t* p, float v)
{
    const unsigned u = __float_as_uint(v);
    *p = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);  // round to nearest even
}
__device__ __forceinline__ void store_out(float* p, float v) { *p = v; }

__device__ __forceinline__ double group16_sum(double v)
{
    v += __shfl_xor(v, 1);
    v += __shfl_xor(v, 2);
    v += __shfl_xor(v, 4);
    v += __shfl_xor(v, 8);
    return v;
}

__global__ void decode_init_kernel(double* anchor_k, double* anchor_v, long long n_anchor,
                                   int32_t* seen, int32_t* skipped, float* tau, int32_t* cache_len,
                                   int32_t* overflow, int B, float tau0)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_anchor) { anchor_k[i] = 0.0; anchor_v[i] = 0.0; }
    if (i < B) { seen[i] = 0; skipped[i] = 0; tau[i] = tau0; cache_len[i] = 0; overflow[i] = 0; }
}

// One workgroup per batch row; a 16-lane group per (tensor, KV head) pair, eight columns a lane.
// The float operations of the threshold rule are the ones of the batched online decision, in
// the same order, with contraction switched off, so both forms agree bit for bit.
// Latency is what this kernel costs, so the row's scalars are fetched up front by the lane
// that needs them, the head statistics are reduced by one wave rather than one lane, and the
// first pair of a group stays in registers for the anchor update.
#pragma clang fp contract(off)
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int s = 1; s < 64; s *= 2) v += __shfl_xor(v, s);
    return v;
}

template <typename T>
__global__ __launch_bounds__(1024) void decode_score_kernel(
    const T* __restrict__ k, const T* __restrict__ v, double* __restrict__ anchor_k,
    double* __restrict__ anchor_v, int32_t* __restrict__ seen, int32_t* __restrict__ skipped,
    float* __restrict__ tau, int32_t* __restrict__ cache_len, int32_t* __restrict__ overflow,
    T* __restrict__ k_cache, T* __restrict__ v_cache, int capacity, int Hkv, int ema, double gamma,
    int inclusive, int fusion, int warmup, float target, float eta,
    uint8_t* __restrict__ skip_out, float* __restrict__ fused_out)
{
    __shared__ double cosb[2][128];
    __shared__ int slot_s;
    const int b = blockIdx.x;
    const int grp = threadIdx.x >> 4, c8 = threadIdx.x & 15, n_grp = blockDim.x >> 4;
    const int t = seen[b];
    int n_skipped = 0, len = 0;
    float th_old = 0.f;
    if (threadIdx.x == 0) { n_skipped = skipped[b]; len = cache_len[b]; th_old = tau[b]; }
    // the anchor a row is compared with is f_a * state + f_x * row
    const int rows_in = inclusive ? t + 1 : t;
    const double f_a = ema ? (inclusive ? gamma : 1.0) : (rows_in > 0 ? 1.0 / (double)rows_in : 0.0);
    const double f_x = inclusive ? (ema ? 1.0 - gamma : f_a) : 0.0;

    float x0[8];       // the group's first pair, kept for the update below
    double a0[8];
    for (int pr = grp; pr < 2 * Hkv; pr += n_grp) {
        const int w = pr >= Hkv, h = pr - w * Hkv;
        const long long off = ((long long)b * Hkv + h) * kHeadDim + c8 * 8;
        float x[8];
        load8((w ? v : k) + off, x);
        const double* a = (w ? anchor_v : anchor_k) + off;
        double av[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) av[c] = a[c];
        if (pr == grp) {
#pragma unroll
            for (int c = 0; c < 8; ++c) { x0[c] = x[c]; a0[c] = av[c]; }
        }
        double dot = 0.0, na = 0.0, nx = 0.0;
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            const double ac = av[c] * f_a + (double)x[c] * f_x;
            dot += ac * (double)x[c];
            na += ac * ac;
            nx += (double)x[c] * (double)x[c];
        }
        dot = group16_sum(dot); na = group16_sum(na); nx = group16_sum(nx);
        double den = sqrt(na) * sqrt(nx);
        den = den < kEpsCos ? kEpsCos : den;
        double cs = dot / den;
        cs = cs > 1.0 ? 1.0 : (cs < -1.0 ? -1.0 : cs);
        if (c8 == 0) cosb[w][h] = cs;
    }
    __syncthreads();  // every read of seen[b] above precedes lane 0's update below

    if (threadIdx.x < 64) {
        // mean and population variance over the heads (two passes), one wave
        const int l = threadIdx.x;
        const double ck0 = l < Hkv ? cosb[0][l] : 0.0, cv0 = l < Hkv ? cosb[1][l] : 0.0;
        const double ck1 = l + 64 < Hkv ? cosb[0][l + 64] : 0.0, cv1 = l + 64 < Hkv ? cosb[1][l + 64] : 0.0;
        const double sk = wave_sum(ck0 + ck1) / (double)Hkv, sv = wave_sum(cv0 + cv1) / (double)Hkv;
        double dk = 0.0, dv = 0.0;
        if (l < Hkv) { dk = (ck0 - sk) * (ck0 - sk); dv = (cv0 - sv) * (cv0 - sv); }
        if (l + 64 < Hkv) { dk += (ck1 - sk) * (ck1 - sk); dv += (cv1 - sv) * (cv1 - sv); }
        const double ek = wave_sum(dk) / (double)Hkv + kEpsVar, ev = wave_sum(dv) / (double)Hkv + kEpsVar;
        if (l == 0) {
            const double alpha = fusion == 0 ? (1.0 / ev) / (1.0 / ek + 1.0 / ev)
                               : fusion == 1 ? (1.0 / ek) / (1.0 / ek + 1.0 / ev)
                               : fusion == 2 ? 1.0 : 0.0;
            const float S = (float)(alpha * sk + (1.0 - alpha) * sv);

            const float inv = t == 0 ? 0.0f : 1.0f / (float)t;
            const float p_current = (float)n_skipped * inv;
            const float diff = p_current - target;
            const float th = fmaf(eta, diff, th_old);
            int skip = (t >= warmup) && (S > th);
            int slot = -1;
            if (!skip) {
                if (len >= capacity) { overflow[b] = 1; skip = 1; }  // handled as skipped
                else { slot = len; cache_len[b] = len + 1; }
            }
            tau[b] = th;
            seen[b] = t + 1;
            skipped[b] = n_skipped + skip;
            skip_out[b] = (uint8_t)skip;
            fused_out[b] = S;
            slot_s = slot;
        }
    }
    __syncthreads();
    const int slot = slot_s;

    for (int pr = grp; pr < 2 * Hkv; pr += n_grp) {
        const int w = pr >= Hkv, h = pr - w * Hkv;
        const long long off = ((long long)b * Hkv + h) * kHeadDim + c8 * 8;
        const T* src = (w ? v : k) + off;
        double* a = (w ? anchor_v : anchor_k) + off;
        float x[8];
        double av[8];
        if (pr == grp) {
#pragma unroll
            for (int c = 0; c < 8; ++c) { x[c] = x0[c]; av[c] = a0[c]; }
        } else {
            load8(src, x);
#pragma unroll
            for (int c = 0; c < 8; ++c) av[c] = a[c];
        }
#pragma unroll
        for (int c = 0; c < 8; ++c)
            a[c] = ema ? gamma * av[c] + (1.0 - gamma) * (double)x[c] : av[c] + (double)x[c];
        if (slot >= 0)
            copy8((w ? v_cache : k_cache) + (((long long)b * Hkv + h) * capacity + slot) * kHeadDim + c8 * 8, src);
    }
}
#pragma clang fp contract(fast)

// Attention of the new token over one slice of its row's cache, for the G query heads that
// share a KV head.  A 16-lane group owns every 16th key of the slice and keeps its own running
// (max, sum, numerators); groups are merged through shuffles and LDS, the slices by
// decode_merge_kernel.  Partial result per (row, query head, slice): kPartStride floats.
template <typename T, int G>
__global__ __launch_bounds__(256) void decode_attend_kernel(
    const T* __restrict__ q, const T* __restrict__ k_cache, const T* __restrict__ v_cache,
    const int32_t* __restrict__ cache_len, const uint8_t* __restrict__ skip,
    float* __restrict__ part, int Hq, int Hkv, int capacity, int n_split, float scale_log2e)
{
    __shared__ float merge[4][G][kPartStride];
    const int sp = blockIdx.x % n_split;
    const int hg = (blockIdx.x / n_split) % (Hq / G);  // group of G query heads
    const int b = blockIdx.x / n_split / (Hq / G);
    if (skip[b]) return;  // the merge kernel writes the zero row
    const int hq0 = hg * G, hk = hq0 / (Hq / Hkv);
    const int len = cache_len[b];
    int chunk = (len + n_split - 1) / n_split;
    chunk = (chunk + 15) & ~15;
    const int lo = sp * chunk, hi = min(len, lo + chunk);
    const int grp = threadIdx.x >> 4, c8 = threadIdx.x & 15, wave = threadIdx.x >> 6;

    float qf[G][8], acc[G][8], mx[G], sum[G];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        load8(q + ((long long)b * Hq + hq0 + g) * kHeadDim + c8 * 8, qf[g]);
#pragma unroll
        for (int c = 0; c < 8; ++c) { qf[g][c] *= scale_log2e; acc[g][c] = 0.f; }
        mx[g] = kLowest; sum[g] = 0.f;
    }
    const long long row0 = ((long long)b * Hkv + hk) * capacity;
    const T* kb = k_cache + row0 * kHeadDim + c8 * 8;
    const T* vb = v_cache + row0 * kHeadDim + c8 * 8;

    for (int j = lo + grp; j < hi; j += 64) {
        float kk[4][8], vv[4][8];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int ju = min(j + 16 * u, hi - 1);  // a valid row; its score is discarded below
            load8(kb + (long long)ju * kHeadDim, kk[u]);
            load8(vb + (long long)ju * kHeadDim, vv[u]);
        }
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float s[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                float d = 0.f;
#pragma unroll
                for (int c = 0; c < 8; ++c) d = fmaf(qf[g][c], kk[u][c], d);
                d = row16_sum(d);
                s[u] = (j + 16 * u < hi) ? d : kLowest;
            }
            const float m_new = fmaxf(fmaxf(mx[g], fmaxf(s[0], s[1])), fmaxf(s[2], s[3]));
            const float scale_old = exp2f(mx[g] - m_new);
            float p[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) p[u] = exp2f(s[u] - m_new);
            sum[g] = fmaf(sum[g], scale_old, (p[0] + p[1]) + (p[2] + p[3]));
#pragma unroll
            for (int c = 0; c < 8; ++c) {
                float a = acc[g][c] * scale_old;
#pragma unroll
                for (int u = 0; u < 4; ++u) a = fmaf(p[u], vv[u][c], a);
                acc[g][c] = a;
            }
            mx[g] = m_new;
        }
    }

    // merge the four groups of a wave (lanes 16 and 32 apart), then the four waves through LDS
#pragma unroll
    for (int g = 0; g < G; ++g) {
#pragma unroll
        for (int step = 16; step <= 32; step *= 2) {
            const float m_o = __shfl_xor(mx[g], step);
            const float m_new = fmaxf(mx[g], m_o);
            const float w_me = exp2f(mx[g] - m_new), w_o = exp2f(m_o - m_new);
            sum[g] = sum[g] * w_me + __shfl_xor(sum[g], step) * w_o;
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[g][c] = acc[g][c] * w_me + __shfl_xor(acc[g][c], step) * w_o;
            mx[g] = m_new;
        }
        if ((threadIdx.x & 63) < 16) {
#pragma unroll
            for (int c = 0; c < 8; ++c) merge[wave][g][c8 * 8 + c] = acc[g][c];
            if (c8 == 0) { merge[wave][g][kHeadDim] = mx[g]; merge[wave][g][kHeadDim + 1] = sum[g]; }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < G * kPartStride; i += blockDim.x) {
        const int g = i / kPartStride, c = i - g * kPartStride;
        float m_all = kLowest;
#pragma unroll
        for (int w = 0; w < 4; ++w) m_all = fmaxf(m_all, merge[w][g][kHeadDim]);
        float out;
        if (c == kHeadDim) {
            out = m_all;
        } else {
            out = 0.f;
#pragma unroll
            for (int w = 0; w < 4; ++w) out = fmaf(merge[w][g][c], exp2f(merge[w][g][kHeadDim] - m_all), out);
        }
        part[(((long long)b * Hq + hq0 + g) * n_split + sp) * kPartStride + c] = out;
    }
}

// One workgroup of 128 threads per (row, query head): weighted sum of the slices' partial
// results, or the zero row of a skipped token.
template <typename T>
__global__ __launch_bounds__(128) void decode_merge_kernel(const float* __restrict__ part,
                                                           const uint8_t* __restrict__ skip,
                                                           T* __restrict__ o, int Hq, int n_split)
{
    const int b = blockIdx.x / Hq;
    const int c = threadIdx.x;
    T* out = o + (long long)blockIdx.x * kHeadDim + c;
    if (skip[b]) { store_out(out, 0.f); return; }
    const float* pr = part + (long long)blockIdx.x * n_split * kPartStride;
    float m_all = kLowest;
    for (int s = 0; s < n_split; ++s) m_all = fmaxf(m_all, pr[s * kPartStride + kHeadDim]);
    float num = 0.f, den = 0.f;
    for (int s = 0; s < n_split; ++s) {
        const float w = exp2f(pr[s * kPartStride + kHeadDim] - m_all);
        num = fmaf(pr[s * kPartStride + c], w, num);
        den = fmaf(pr[s * kPartStride + kHeadDim + 1], w, den);
    }
    store_out(out, num / den);
}

// Hand-off from the batched path: the anchors as they stand after all n rows of a prompt.
// One workgroup per (tensor, batch row, KV head); a 16-lane group folds every 16th row in
// Horner form, A <- g^16 A + x (g = 1 for the exact mean, whose state is the plain sum), brings
// its partial to the end of the prompt with g^(rows after its last one), and the 16 partials
// are added through LDS.  All in double.  Rows further back than `window` from the end are
// skipped (the incremental anchor forgets them: g^window is far below double resolution).
template <typename T>
__global__ __launch_bounds__(256) void decode_seed_anchor_kernel(
    const T* __restrict__ K, const T* __restrict__ V, double* __restrict__ anchor_k,
    double* __restrict__ anchor_v, int Hkv, int n, long long s_b, long long s_h, long long s_t,
    double g, double weight, int window)
{
    __shared__ double part[16][kHeadDim];
    const int w = blockIdx.x & 1, bh = blockIdx.x >> 1;
    const int b = bh / Hkv, h = bh % Hkv;
    const int grp = threadIdx.x >> 4, c8 = threadIdx.x & 15;
    const T* X = (w ? V : K) + b * s_b + h * s_h + c8 * 8;
    double g16 = g;
#pragma unroll
    for (int i = 0; i < 4; ++i) g16 *= g16;
    double a[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) a[c] = 0.0;
    const int j0 = (n - window > 0 ? n - window : 0);
    int last = -1;
    for (int j = j0 + grp; j < n; j += 16) {
        float x[8];
        load8(X + (long long)j * s_t, x);
#pragma unroll
        for (int c = 0; c < 8; ++c) a[c] = g16 * a[c] + (double)x[c];
        last = j;
    }
    double tail = weight;  // weight * g^(n - 1 - last)
    for (int i = last; last >= 0 && i < n - 1; ++i) tail *= g;
#pragma unroll
    for (int c = 0; c < 8; ++c) part[grp][c8 * 8 + c] = last >= 0 ? a[c] * tail : 0.0;
    __syncthreads();
    if (threadIdx.x < kHeadDim) {
        double sum = 0.0;
#pragma unroll
        for (int q = 0; q < 16; ++q) sum += part[q][threadIdx.x];
        (w ? anchor_v : anchor_k)[(long long)bh * kHeadDim + threadIdx.x] = sum;
    }
}

// Hand-off from the batched path: the kept rows of K and V, in order, into the caches, and
// the controller's counters.  Grid: (row blocks of 16, batch * KV heads).
template <typename T>
__global__ __launch_bounds__(256) void decode_seed_cache_kernel(
    const T* __restrict__ K, const T* __restrict__ V, const int32_t* __restrict__ kept_idx,
    const int32_t* __restrict__ count, T* __restrict__ k_cache, T* __restrict__ v_cache,
    int32_t* __restrict__ seen, int32_t* __restrict__ skipped, int32_t* __restrict__ cache_len,
    int32_t* __restrict__ overflow, int Hkv, int n, int capacity, long long s_b, long long s_h,
    long long s_t)
{
    const int bh = blockIdx.y, b = bh / Hkv, h = bh % Hkv;
    const int m = count[b];
    if (blockIdx.x == 0 && h == 0 && threadIdx.x == 0) {
        seen[b] = n; skipped[b] = n - m; cache_len[b] = m; overflow[b] = 0;
    }
    const int i = blockIdx.x * 16 + (threadIdx.x >> 4), c8 = threadIdx.x & 15;
    if (i >= m) return;
    const long long src = b * s_b + h * s_h + (long long)kept_idx[(long long)b * n + i] * s_t + c8 * 8;
    const long long dst = ((long long)bh * capacity + i) * kHeadDim + c8 * 8;
    copy8(k_cache + dst, K + src);
    copy8(v_cache + dst, V + src);
}

template <typename T>
hipError_t launch_decode_seed_t(const DecodeArgs& a, const T* K, const T* V, const int32_t* kept_idx,
                                const int32_t* count, int n, const long long* kvs, hipStream_t s)
{
    const double g = a.ema ? a.gamma : 1.0;
    // rows that still matter to the incremental anchor: g^window <= 1e-40
    int window = n;
    if (a.ema) {
        const double rows = g > 0.0 ? ceil(-92.2 / log(g)) : 1.0;
        window = rows < (double)n ? (int)rows : n;
    }
    decode_seed_anchor_kernel<T><<<dim3(2 * a.B * a.Hkv), dim3(256), 0, s>>>(
        K, V, a.anchor_k, a.anchor_v, a.Hkv, n, kvs[0], kvs[1], kvs[2], g, a.ema ? 1.0 - a.gamma : 1.0, window);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    decode_seed_cache_kernel<T><<<dim3((n + 15) / 16, a.B * a.Hkv), dim3(256), 0, s>>>(
        K, V, kept_idx, count, (T*)a.k_cache, (T*)a.v_cache, a.seen, a.skipped, a.cache_len, a.overflow,
        a.Hkv, n, a.capacity, kvs[0], kvs[1], kvs[2]);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_decode_step_t(const DecodeArgs& a, const T* q, const T* k, const T* v, T* o,
                                hipStream_t s)
{
    const int threads = std::min(1024, (32 * a.Hkv + 63) / 64 * 64);  // 16 lanes per (tensor, head)
    decode_score_kernel<T><<<dim3(a.B), dim3(threads), 0, s>>>(
        k, v, a.anchor_k, a.anchor_v, a.seen, a.skipped, a.tau, a.cache_len, a.overflow,
        (T*)a.k_cache, (T*)a.v_cache, a.capacity, a.Hkv, a.ema, a.gamma, a.inclusive, a.fusion, a.warmup,
        a.target, a.eta, a.skip, a.fused);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int group = a.Hq / a.Hkv;
    const float sl2 = a.scale * 1.4426950408889634f;
#define TF_DECODE_ATTEND(G)                                                                       \
    decode_attend_kernel<T, G><<<dim3(a.B * (a.Hq / G) * a.n_split), dim3(256), 0, s>>>(          \
        q, (const T*)a.k_cache, (const T*)a.v_cache, a.cache_len, a.skip, a.part, a.Hq, a.Hkv,     \
        a.capacity, a.n_split, sl2)
    if (group == 8) TF_DECODE_ATTEND(8);
    else if (group == 4) TF_DECODE_ATTEND(4);
    else if (group == 2) TF_DECODE_ATTEND(2);
    else TF_DECODE_ATTEND(1);  // other ratios: one query head per workgroup
#undef TF_DECODE_ATTEND
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    decode_merge_kernel<T><<<dim3(a.B * a.Hq), dim3(128), 0, s>>>(a.part, a.skip, o, a.Hq, a.n_split);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode_init(const DecodeArgs& a, float tau0, hipStream_t s)
{
    const long long n_anchor = (long long)a.B * a.Hkv * kHeadDim;
    const long long n = std::max<long long>(n_anchor, a.B);
    decode_init_kernel<<<dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s>>>(
        a.anchor_k, a.anchor_v, n_anchor, a.seen, a.skipped, a.tau, a.cache_len, a.overflow, a.B, tau0);
    return hipGetLastError();
}

hipError_t launch_decode_seed(const DecodeArgs& a, int dtype, const void* K, const void* V,
                              const int32_t* kept_idx, const int32_t* count, int n,
                              const long long* kvs, hipStream_t s)
{
    if (dtype == 0) return launch_decode_seed_t<float>(a, (const float*)K, (const float*)V, kept_idx, count, n, kvs, s);
    return launch_decode_seed_t<uint16_t>(a, (const uint16_t*)K, (const uint16_t*)V, kept_idx, count, n, kvs, s);
}

hipError_t launch_decode_step(const DecodeArgs& a, int dtype, const void* q, const void* k,
                              const void* v, void* o, hipStream_t s)
{
    if (dtype == 0)
        return launch_decode_step_t<float>(a, (const float*)q, (const float*)k, (const float*)v, (float*)o, s);
    return launch_decode_step_t<uint16_t>(a, (const uint16_t*)q, (const uint16_t*)k,
                                          (const uint16_t*)v, (uint16_t*)o, s);
}

}  // namespace tf
