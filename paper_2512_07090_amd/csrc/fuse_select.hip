// Head statistics and variance-aware fusion (Algorithm 1 mean/var/alpha/s_KV lines; Eq. 2),
// the exact-count keep decision (Algorithm 1 "skip if s_KV > tau" with tau placed so that
// exactly m tokens stay), and stream compaction of the kept positions.
#include "tf_kernels.h"

namespace tf {

namespace {

// ------------------------------------------------------------------------------ fusion
// 64 tokens per workgroup.  All 256 threads stage the tokens' per-head cosines in LDS
// ([head][token]: global reads and LDS accesses are unit-stride across a wave; four head
// groups load in parallel so enough loads are in flight); then one thread per token takes the
// mean and the two-pass variance over the heads (the head count is a run-time value).
constexpr int kFuseTokens = 64;
constexpr int kFuseThreads = 256;

__global__ __launch_bounds__(kFuseThreads) void fuse_kernel(const float* __restrict__ sim_k,
                                                            const float* __restrict__ sim_v,
                                                            int H, int n, int mode,
                                                            float* __restrict__ fused)
{
    extern __shared__ float stage[];  // [2][H][kFuseTokens]
    float* ck = stage;
    float* cv = stage + (size_t)H * kFuseTokens;
    const int b = blockIdx.y;
    const int tok = threadIdx.x & (kFuseTokens - 1);
    const int hg = threadIdx.x / kFuseTokens;
    const int t = blockIdx.x * kFuseTokens + tok;
    if (t < n) {
        // key-only / value-only scores read one tensor's cosines (the other was not computed)
        const float* pk = (mode == 3 ? sim_v : sim_k) + (long long)b * H * n + t;
        const float* pv = (mode == 2 ? sim_k : sim_v) + (long long)b * H * n + t;
        for (int h = hg; h < H; h += kFuseThreads / kFuseTokens) {
            ck[h * kFuseTokens + tok] = pk[(long long)h * n];
            cv[h * kFuseTokens + tok] = pv[(long long)h * n];
        }
    }
    __syncthreads();
    if (hg != 0 || t >= n) return;
    float sk = 0.f, sv = 0.f;
    for (int h = 0; h < H; ++h) {
        sk += ck[h * kFuseTokens + tok];
        sv += cv[h * kFuseTokens + tok];
    }
    const float inv_h = 1.0f / (float)H;
    sk *= inv_h;
    sv *= inv_h;
    float vk = 0.f, vv = 0.f;
    for (int h = 0; h < H; ++h) {
        const float dk = ck[h * kFuseTokens + tok] - sk;
        const float dv = cv[h * kFuseTokens + tok] - sv;
        vk = fmaf(dk, dk, vk);
        vv = fmaf(dv, dv, vv);
    }
    const float ek = vk * inv_h + 1e-12f, ev = vv * inv_h + 1e-12f;
    float alpha;
    if (mode == 0)
        alpha = ek / (ek + ev);  // = (1/ev) / (1/ek + 1/ev), the printed form of Eq. 2
    else if (mode == 1)
        alpha = ev / (ek + ev);  // = (1/ek) / (1/ek + 1/ev)
    else
        alpha = mode == 2 ? 1.f : 0.f;
    fused[(long long)b * n + t] = alpha * sk + (1.f - alpha) * sv;
}

// ------------------------------------------------------------------------------ block scan
constexpr int kSelThreads = 1024;
constexpr int kSelWaves = kSelThreads / 64;

// Exclusive prefix sum of one int per thread over the 1024-thread block; *total gets the
// block sum.  `lds` must hold kSelWaves + 1 ints.  Ends with a barrier, so `lds` may be
// reused immediately.
__device__ __forceinline__ int block_excl_scan(int v, int* lds, int* total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const int o = __shfl_up(inc, off);
        if (lane >= off) inc += o;
    }
    if (lane == 63) lds[wave] = inc;
    __syncthreads();
    int base = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < kSelWaves; ++w) {
        const int x = lds[w];
        if (w < wave) base += x;
        tot += x;
    }
    __syncthreads();
    *total = tot;
    return base + inc - v;
}

// Order-preserving map from float to unsigned; -0 is folded onto +0 so that the two compare
// equal, as they do as floats (ties then go by index).
__device__ __forceinline__ unsigned f2key(float f)
{
    unsigned u = __builtin_bit_cast(unsigned, f);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key2f(unsigned k)
{
    const unsigned u = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
    return __builtin_bit_cast(float, u);
}

// ------------------------------------------------------------------------------ decision
// One workgroup per batch row.  The `want`-th smallest score among the non-forced tokens is
// found by a most-significant-digit-first radix select on the order-preserving keys (four
// passes of 8 bits, a 256-bin LDS histogram each); tokens strictly below it are kept, tokens
// equal to it are kept in index order until the count is met.
__global__ __launch_bounds__(kSelThreads) void select_kernel(const float* __restrict__ fused,
                                                             int n, int m, int warmup,
                                                             uint8_t* __restrict__ keep,
                                                             float* __restrict__ tau)
{
    __shared__ int hist[256];
    __shared__ int scan_lds[kSelWaves + 1];
    __shared__ unsigned sel_prefix;
    __shared__ int sel_k;

    const int b = blockIdx.x;
    const float* S = fused + (long long)b * n;
    uint8_t* kp = keep + (long long)b * n;
    const int tid = threadIdx.x;
    const int forced = min(max(warmup, 0), m);
    const int want = m - forced;

    if (m >= n || want <= 0) {
        for (int t = tid; t < n; t += kSelThreads) kp[t] = (m >= n || t < forced) ? 1 : 0;
        if (tid == 0 && tau) tau[b] = m >= n ? INFINITY : -INFINITY;
        return;
    }

    unsigned prefix = 0;
    int k = want;  // 1-based rank still to find inside the current prefix bucket
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        const unsigned himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int t = forced + tid; t < n; t += kSelThreads) {
            const unsigned key = f2key(S[t]);
            if ((key & himask) == prefix) atomicAdd(&hist[(key >> shift) & 255u], 1);
        }
        __syncthreads();
        const int cnt = tid < 256 ? hist[tid] : 0;
        int total;
        const int before = block_excl_scan(cnt, scan_lds, &total);
        if (tid < 256 && before < k && k <= before + cnt) {
            sel_prefix = prefix | ((unsigned)tid << shift);
            sel_k = k - before;
        }
        __syncthreads();
        prefix = sel_prefix;
        k = sel_k;
        __syncthreads();
    }
    const unsigned tkey = prefix;  // key of the want-th smallest score
    const int k_eq = k;            // how many tokens equal to it are kept (>= 1)
    if (tid == 0 && tau) tau[b] = key2f(tkey);

    int eq_base = 0;
    for (int t0 = forced; t0 < n; t0 += kSelThreads) {
        const int t = t0 + tid;
        unsigned key = 0xffffffffu;
        if (t < n) key = f2key(S[t]);
        const int is_eq = (t < n && key == tkey) ? 1 : 0;
        int total;
        const int rank = eq_base + block_excl_scan(is_eq, scan_lds, &total);
        eq_base += total;
        if (t < n) kp[t] = (key < tkey || (is_eq && rank < k_eq)) ? 1 : 0;
    }
    for (int t = tid; t < forced; t += kSelThreads) kp[t] = 1;
}

// ------------------------------------------------------------------------------ compaction
// One workgroup per batch row: ordered exclusive prefix count of the keep flags, kept
// positions written ascending.
__global__ __launch_bounds__(kSelThreads) void compact_kernel(const uint8_t* __restrict__ keep,
                                                              int n, int m,
                                                              int32_t* __restrict__ kept_idx)
{
    __shared__ int scan_lds[kSelWaves + 1];
    const int b = blockIdx.x;
    const uint8_t* kp = keep + (long long)b * n;
    int32_t* out = kept_idx + (long long)b * m;
    int base = 0;
    for (int t0 = 0; t0 < n; t0 += kSelThreads) {
        const int t = t0 + threadIdx.x;
        const int flag = (t < n && kp[t]) ? 1 : 0;
        int total;
        const int pos = base + block_excl_scan(flag, scan_lds, &total);
        base += total;
        if (flag && pos < m) out[pos] = t;
    }
}

// ------------------------------------------------------------------------------ decision + compaction
// Same decision as select_kernel followed by compact_kernel, in one launch, for rows of up to
// 1024 * IPT tokens: a thread keeps its IPT consecutive scores in registers, so the four radix
// passes and the two ordered scans (rank among the threshold's equals, rank among the kept)
// touch only registers and LDS.
template <int IPT>
__global__ __launch_bounds__(kSelThreads) void select_compact_kernel(
    const float* __restrict__ fused, int n, int m, int warmup, uint8_t* __restrict__ keep,
    int32_t* __restrict__ kept_idx, float* __restrict__ tau)
{
    __shared__ int hist[256];
    __shared__ int scan_lds[kSelWaves + 1];
    __shared__ unsigned sel_prefix;
    __shared__ int sel_k;

    const int b = blockIdx.x;
    const float* S = fused + (long long)b * n;
    uint8_t* kp = keep + (long long)b * n;
    int32_t* out = kept_idx + (long long)b * m;
    const int tid = threadIdx.x;
    const int t0 = tid * IPT;
    const int forced = min(max(warmup, 0), m);
    const int want = m - forced;
    const bool all = m >= n;            // nothing is filtered
    const bool none = want <= 0;        // no non-forced token is kept

    // keys of this thread's tokens; forced tokens and the tail past n take no part in the
    // selection (cand = false)
    unsigned key[IPT];
    bool cand[IPT];
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int t = t0 + i;
        cand[i] = t >= forced && t < n;
        key[i] = cand[i] ? f2key(S[t]) : 0xffffffffu;
    }

    unsigned tkey = 0;
    int k_eq = 0;
    if (!all && !none) {
        unsigned prefix = 0;
        int k = want;  // 1-based rank still to find inside the current prefix bucket
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            const unsigned himask = pass == 0 ? 0u : (0xffffffffu << (shift + 8));
            if (tid < 256) hist[tid] = 0;
            __syncthreads();
            // a thread's consecutive tokens that fall into the same bin share one atomic: scores
            // are cosines, so in the first passes nearly all of them do, and colliding atomics
            // are what this loop costs
            int run_bin = -1, run_len = 0;
#pragma unroll
            for (int i = 0; i < IPT; ++i) {
                if (cand[i] && (key[i] & himask) == prefix) {
                    const int bin = (int)((key[i] >> shift) & 255u);
                    if (bin != run_bin) {
                        if (run_len) atomicAdd(&hist[run_bin], run_len);
                        run_bin = bin;
                        run_len = 0;
                    }
                    ++run_len;
                }
            }
            if (run_len) atomicAdd(&hist[run_bin], run_len);
            __syncthreads();
            const int cnt = tid < 256 ? hist[tid] : 0;
            int total;
            const int before = block_excl_scan(cnt, scan_lds, &total);
            if (tid < 256 && before < k && k <= before + cnt) {
                sel_prefix = prefix | ((unsigned)tid << shift);
                sel_k = k - before;
            }
            __syncthreads();
            prefix = sel_prefix;
            k = sel_k;
            __syncthreads();
        }
        tkey = prefix;
        k_eq = k;
    }
    if (tid == 0 && tau) tau[b] = all ? INFINITY : (none ? -INFINITY : key2f(tkey));

    // rank of this thread's threshold-equal tokens among all of them, in index order
    int n_eq = 0;
#pragma unroll
    for (int i = 0; i < IPT; ++i) n_eq += (cand[i] && !all && !none && key[i] == tkey) ? 1 : 0;
    int total_eq;
    int eq_rank = block_excl_scan(n_eq, scan_lds, &total_eq);

    bool kept[IPT];
    int n_kept = 0;
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int t = t0 + i;
        bool kflag;
        if (t >= n)
            kflag = false;
        else if (all || t < forced)
            kflag = true;
        else if (none)
            kflag = false;
        else if (key[i] < tkey)
            kflag = true;
        else if (key[i] == tkey)
            kflag = eq_rank++ < k_eq;
        else
            kflag = false;
        kept[i] = kflag;
        n_kept += kflag ? 1 : 0;
    }
    int total_kept;
    int pos = block_excl_scan(n_kept, scan_lds, &total_kept);
#pragma unroll
    for (int i = 0; i < IPT; ++i) {
        const int t = t0 + i;
        if (t < n) kp[t] = kept[i] ? 1 : 0;
        if (kept[i]) {
            if (pos < m) out[pos] = t;
            ++pos;
        }
    }
}

// ------------------------------------------------------------------------------ online decision
// Adaptive threshold (Algorithm 1 threshold / skip lines, warm-up of Section 3.2, Eq. 4): a
// sequential recurrence over a row's tokens,
//   tau <- fma(eta, (float)skipped * (1 / t) - target, tau);  skip iff t >= W and S_t > tau,
// all in float so that the result is reproducible bit for bit.  One workgroup per batch row
// walks the row in chunks of kOnChunk tokens: all threads stage the chunk's scores and the
// reciprocals 1 / t in LDS, thread 0 runs the recurrence and leaves the running count of
// skipped tokens in place of the scores, then all threads read the decisions off the counts
// and compact them.
constexpr int kOnChunk = 4096;

__global__ __launch_bounds__(kSelThreads) void select_online_kernel(
    const float* __restrict__ fused, int n, int warmup, float target, float eta, float tau0,
    uint8_t* __restrict__ keep, int32_t* __restrict__ kept_idx, int32_t* __restrict__ count,
    float* __restrict__ tau_out)
{
    // every product and difference below is rounded on its own (the only fused operations are
    // the fmaf calls): the recurrence is defined operation by operation
#pragma clang fp contract(off)
    __shared__ __attribute__((aligned(16))) float s_lds[kOnChunk];
    __shared__ __attribute__((aligned(16))) float inv_lds[kOnChunk];
    __shared__ int scan_lds[kSelWaves + 1];
    __shared__ float skip_base;  // skipped tokens before the current chunk

    const int b = blockIdx.x;
    const int tid = threadIdx.x;
    const float* S = fused + (long long)b * n;
    uint8_t* kp = keep + (long long)b * n;
    int32_t* out = kept_idx + (long long)b * n;

    // state of the recurrence (meaningful in thread 0): tau is the threshold token t0 of the
    // next chunk will be judged with, already updated for it
    float skipped = 0.f;  // exact in float up to 2^24 tokens
    float tau = fmaf(eta, 0.f - target, tau0);
    float tau_judged = tau;  // the threshold the latest token was judged with
    int base = 0;            // kept tokens so far
    for (int t0 = 0; t0 < n; t0 += kOnChunk) {
        const int len = min(kOnChunk, n - t0);
        // (warm-up tokens and the padding up to a multiple of 8 get a score that is never above
        // the threshold, so the chain below needs no test for them)
        for (int i = tid; i < ((len + 7) & ~7); i += kSelThreads)
            s_lds[i] = (i < len && t0 + i >= warmup) ? S[t0 + i] : -INFINITY;
        // reciprocal of the NEXT token's index: inv_lds[i] = 1 / (t0 + i + 1)
        for (int i = tid; i < ((len + 7) & ~7); i += kSelThreads) inv_lds[i] = 1.0f / (float)(t0 + i + 1);
        __syncthreads();
        if (tid == 0) {
            // eight tokens at a time: their scores and reciprocals are fetched together (two
            // 16-byte LDS reads each) and the eight steps of the chain run from registers.  A
            // step is five dependent operations (compare, select, multiply, subtract, fma); a
            // lone wave waits about as long for a dependent result as it takes to issue two
            // instructions, so forming both outcomes ahead of the comparison (a shorter chain,
            // twice the instructions) measured slower than this plain form.  The running count
            // of skipped tokens replaces the scores in LDS: the other threads read the
            // decisions off it afterwards (a token was skipped iff the count moved).
            skip_base = skipped;
            for (int i0 = 0; i0 < len; i0 += 8) {
                float sv[8], iv[8], sk[8];
                *reinterpret_cast<float4*>(&sv[0]) = *reinterpret_cast<const float4*>(&s_lds[i0]);
                *reinterpret_cast<float4*>(&sv[4]) = *reinterpret_cast<const float4*>(&s_lds[i0 + 4]);
                *reinterpret_cast<float4*>(&iv[0]) = *reinterpret_cast<const float4*>(&inv_lds[i0]);
                *reinterpret_cast<float4*>(&iv[4]) = *reinterpret_cast<const float4*>(&inv_lds[i0 + 4]);
                float tau_in[8];  // the threshold each of the eight tokens is judged with
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    tau_in[u] = tau;
                    const float s1 = skipped + 1.f;
                    skipped = sv[u] > tau ? s1 : skipped;
                    const float p_next = skipped * iv[u];
                    const float diff = p_next - target;
                    tau = fmaf(eta, diff, tau);
                    sk[u] = skipped;
                }
                *reinterpret_cast<float4*>(&s_lds[i0]) = *reinterpret_cast<const float4*>(&sk[0]);
                *reinterpret_cast<float4*>(&s_lds[i0 + 4]) = *reinterpret_cast<const float4*>(&sk[4]);
                if (i0 + 8 >= len) {  // the group that holds the row's last token
#pragma unroll
                    for (int u = 0; u < 8; ++u)
                        if (t0 + i0 + u == n - 1) tau_judged = tau_in[u];
                }
            }
        }
        __syncthreads();
        for (int i0 = 0; i0 < len; i0 += kSelThreads) {
            const int i = i0 + tid;
            // kept iff the count of skipped tokens did not move at token i
            const int flag = i < len ? (s_lds[i] == (i > 0 ? s_lds[i - 1] : skip_base)) : 0;
            int total;
            const int pos = base + block_excl_scan(flag, scan_lds, &total);
            base += total;
            if (i < len) kp[t0 + i] = (uint8_t)flag;
            if (flag) out[pos] = t0 + i;
        }
        __syncthreads();
    }
    for (int i = base + tid; i < n; i += kSelThreads) out[i] = -1;
    if (tid == 0) {
        count[b] = base;
        if (tau_out) tau_out[b] = tau_judged;
    }
}

__global__ void mask_from_idx_kernel(const int32_t* __restrict__ kept_idx, int n, int m,
                                     uint8_t* __restrict__ keep,
                                     const int32_t* __restrict__ counts, long long idx_stride)
{
    const int b = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (counts ? counts[b] : m)) {
        const int p = kept_idx[(long long)b * idx_stride + i];
        if (p >= 0 && p < n) keep[(long long)b * n + p] = 1;
    }
}

__global__ void clear_bytes_kernel(uint8_t* p, long long count)
{
    const long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < count) p[i] = 0;
}

}  // namespace

hipError_t launch_fuse(const Dims& d, int fusion, const float* sim_k, const float* sim_v,
                       float* fused, hipStream_t s)
{
    const size_t lds = (size_t)2 * d.Hkv * kFuseTokens * sizeof(float);
    dim3 grid((d.n + kFuseTokens - 1) / kFuseTokens, d.B);
    fuse_kernel<<<grid, dim3(kFuseThreads), lds, s>>>(sim_k, sim_v, d.Hkv, d.n, fusion, fused);
    return hipGetLastError();
}

hipError_t launch_select(const Dims& d, int warmup, const float* fused, uint8_t* keep,
                         float* tau, hipStream_t s)
{
    select_kernel<<<dim3(d.B), dim3(kSelThreads), 0, s>>>(fused, d.n, d.m, warmup, keep, tau);
    return hipGetLastError();
}

hipError_t launch_select_compact(const Dims& d, int warmup, const float* fused, uint8_t* keep,
                                 int32_t* kept_idx, float* tau, hipStream_t s)
{
    const int ipt = (d.n + kSelThreads - 1) / kSelThreads;
    if (ipt <= 4)
        select_compact_kernel<4><<<dim3(d.B), dim3(kSelThreads), 0, s>>>(fused, d.n, d.m, warmup, keep, kept_idx, tau);
    else if (ipt <= 8)
        select_compact_kernel<8><<<dim3(d.B), dim3(kSelThreads), 0, s>>>(fused, d.n, d.m, warmup, keep, kept_idx, tau);
    else if (ipt <= 32)
        select_compact_kernel<32><<<dim3(d.B), dim3(kSelThreads), 0, s>>>(fused, d.n, d.m, warmup, keep, kept_idx, tau);
    else {
        // longer rows: scores stay in global memory, decision and compaction in two launches
        select_kernel<<<dim3(d.B), dim3(kSelThreads), 0, s>>>(fused, d.n, d.m, warmup, keep, tau);
        compact_kernel<<<dim3(d.B), dim3(kSelThreads), 0, s>>>(keep, d.n, d.m, kept_idx);
    }
    return hipGetLastError();
}

hipError_t launch_select_online(const Dims& d, int warmup, float target, float eta, float tau0,
                                const float* fused, uint8_t* keep, int32_t* kept_idx,
                                int32_t* count, float* tau, hipStream_t s)
{
    select_online_kernel<<<dim3(d.B), dim3(kSelThreads), 0, s>>>(fused, d.n, warmup, target, eta,
                                                                 tau0, keep, kept_idx, count, tau);
    return hipGetLastError();
}

hipError_t launch_compact(const Dims& d, const uint8_t* keep, int32_t* kept_idx, hipStream_t s)
{
    compact_kernel<<<dim3(d.B), dim3(kSelThreads), 0, s>>>(keep, d.n, d.m, kept_idx);
    return hipGetLastError();
}

__global__ void keep_all_kernel(int n, uint8_t* __restrict__ keep, int32_t* __restrict__ kept_idx,
                                float* __restrict__ tau)
{
    const int b = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        keep[(long long)b * n + i] = 1;
        kept_idx[(long long)b * n + i] = i;
    }
    if (tau && i == 0) tau[b] = INFINITY;
}

hipError_t launch_keep_all(const Dims& d, uint8_t* keep, int32_t* kept_idx, float* tau,
                           hipStream_t s)
{
    keep_all_kernel<<<dim3((d.n + 255) / 256, d.B), dim3(256), 0, s>>>(d.n, keep, kept_idx, tau);
    return hipGetLastError();
}

__global__ void keep_none_kernel(int n, uint8_t* __restrict__ keep, float* __restrict__ tau)
{
    const int b = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) keep[(long long)b * n + i] = 0;
    if (tau && i == 0) tau[b] = -INFINITY;
}

hipError_t launch_keep_none(const Dims& d, uint8_t* keep, float* tau, hipStream_t s)
{
    keep_none_kernel<<<dim3((d.n + 255) / 256, d.B), dim3(256), 0, s>>>(d.n, keep, tau);
    return hipGetLastError();
}

hipError_t launch_mask_from_idx(const Dims& d, const int32_t* kept_idx, uint8_t* keep,
                                const int32_t* counts, long long idx_stride, hipStream_t s)
{
    const long long count = (long long)d.B * d.n;
    clear_bytes_kernel<<<dim3((unsigned)((count + 255) / 256)), dim3(256), 0, s>>>(keep, count);
    mask_from_idx_kernel<<<dim3((d.m + 255) / 256, d.B), dim3(256), 0, s>>>(
        kept_idx, d.n, d.m, keep, counts, counts ? idx_stride : (long long)d.m);
    return hipGetLastError();
}

}  // namespace tf
