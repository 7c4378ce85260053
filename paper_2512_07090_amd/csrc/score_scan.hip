// Scoring stage: exclusive prefix sums of K and V along the sequence and, fused with them, the
// per-head cosine of every row with the sum of the rows before it (Algorithm 1, anchor and
// cosine lines; Section 3.2).  cos(mean, x) = cos(sum, x), so the running SUM is carried and
// the 1/t only enters the guard on the denominator.
//
// Work decomposition.  A chain is one (tensor, batch row, KV head): n rows of 128 elements,
// contiguous per row.  A chain is cut into `nseg` segments; one workgroup of 256 threads
// walks one segment in tiles of 128 rows and reads every element exactly once.
//   thread = (row group rg = tid / 16, column slice l = tid % 16); a thread owns 8
//   consecutive rows of the tile and 8 consecutive columns, so a 16-lane DPP row reads one
//   full 256-byte (bf16) row per load and the three 128-long reductions of a row finish
//   inside that DPP row.
//   Two tiles are in flight while a third is processed (three register buffers).
//   Per tile: (1) per-thread column totals of its 8 rows; (2) exclusive scan of those totals
//   over the 16 row groups (bpermute inside a wave, 2 KB of LDS across the 4 waves);
//   (3) each thread replays its 8 rows against its running prefix.
// With nseg > 1 a first kernel reduces every segment but the last to its column totals and
// the scan kernel starts from the sum of the totals before it.
#include "tf_kernels.h"
#include <algorithm>
#include <cmath>

namespace tf {

namespace {

constexpr int kThreads = 256;
constexpr int kR = 8;               // rows per thread per tile
constexpr int kTile = 16 * kR;      // rows per tile

typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <typename T>
struct Row8;

template <>
struct Row8<uint16_t> {             // bf16 storage
    uint4 raw;
    __device__ __forceinline__ void load(const uint16_t* p) { raw = *reinterpret_cast<const uint4*>(p); }
    // the same with the non-temporal hint: the line is not kept in the L2 after this read
    __device__ __forceinline__ void load_streaming(const uint16_t* p)
    {
        const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
        raw = make_uint4(v[0], v[1], v[2], v[3]);
    }
    __device__ __forceinline__ void zero() { raw = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ void unpack(float* x) const
    {
        const unsigned w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __builtin_bit_cast(float, w[i] << 16);
            x[2 * i + 1] = __builtin_bit_cast(float, w[i] & 0xffff0000u);
        }
    }
    // sum of squares of the 8 elements: two exact bf16 products per v_dot2c_f32_bf16
    __device__ __forceinline__ float sumsq() const
    {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        float s = 0.f;
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, raw.x), __builtin_bit_cast(bf16x2, raw.x), s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, raw.y), __builtin_bit_cast(bf16x2, raw.y), s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, raw.z), __builtin_bit_cast(bf16x2, raw.z), s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, raw.w), __builtin_bit_cast(bf16x2, raw.w), s, false);
        return s;
    }
};

template <>
struct Row8<float> {
    float4 lo, hi;
    __device__ __forceinline__ void load(const float* p)
    {
        lo = *reinterpret_cast<const float4*>(p);
        hi = *reinterpret_cast<const float4*>(p + 4);
    }
    __device__ __forceinline__ void load_streaming(const float* p)
    {
        const f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
        const f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p + 4));
        lo = make_float4(a[0], a[1], a[2], a[3]);
        hi = make_float4(b[0], b[1], b[2], b[3]);
    }
    __device__ __forceinline__ void zero() { lo = hi = make_float4(0.f, 0.f, 0.f, 0.f); }
    __device__ __forceinline__ void unpack(float* x) const
    {
        x[0] = lo.x; x[1] = lo.y; x[2] = lo.z; x[3] = lo.w;
        x[4] = hi.x; x[5] = hi.y; x[6] = hi.z; x[7] = hi.w;
    }
    __device__ __forceinline__ float sumsq() const
    {
        float s = lo.x * lo.x;
        s = fmaf(lo.y, lo.y, s); s = fmaf(lo.z, lo.z, s); s = fmaf(lo.w, lo.w, s);
        s = fmaf(hi.x, hi.x, s); s = fmaf(hi.y, hi.y, s); s = fmaf(hi.z, hi.z, s);
        return fmaf(hi.w, hi.w, s);
    }
};

// The 8 rows t_first .. t_first + 7 of a thread, columns col .. col + 7.  Every load is issued
// whatever the row: rows at or past t_end re-read row t_end - 1 (t_end >= 1) and are zeroed by
// clear_rows_past() once they are used, so that no load sits under a branch and the compiler
// can count how many loads are still in flight when it waits for a tile.
// STREAM: the scan reads every row once; loaded with the non-temporal hint, its stream (0.5 GB on
// the benchmark shape) does not displace what the other kernels of the step, and the next launch
// of the scan, find in the caches.  The totals pass, whose rows the scan reads again right
// after, loads them the ordinary way.
template <bool STREAM, typename T>
__device__ __forceinline__ void load_tile(Row8<T>* rows, const T* X, long long s_t, int t_first,
                                          int t_end, int col)
{
#pragma unroll
    for (int r = 0; r < kR; ++r) {
        const int t = min(t_first + r, t_end - 1);
        if (STREAM)
            rows[r].load_streaming(X + (long long)t * s_t + col);
        else
            rows[r].load(X + (long long)t * s_t + col);
    }
}
template <typename T>
__device__ __forceinline__ void clear_rows_past(Row8<T>* rows, int t_first, int t_end)
{
#pragma unroll
    for (int r = 0; r < kR; ++r)
        if (t_first + r >= t_end) rows[r].zero();
}

// One score to global memory.  Written as an instruction of its own so that the compiler's wait
// counting sees loads only: the hardware counts loads and stores in one counter and lets a store
// overtake a load, and with a store possibly in flight the compiler waits for ALL outstanding
// memory operations, the tiles just requested included.  Loads return in order among
// themselves, so "at most k operations outstanding" still means that all but the newest k loads
// have arrived, whether stores are among the outstanding ones or not; nothing in the kernel
// reads a score back.
__device__ __forceinline__ void store_score(float* p, float v)
{
    asm volatile("global_store_dword %0, %1, off" : : "v"(p), "v"(v) : "memory");
}

// Column totals of segments 0..nseg-2 of every chain.
template <typename T>
__global__ __launch_bounds__(kThreads) void segment_totals_kernel(
    const T* __restrict__ K, const T* __restrict__ V, long long s_b, long long s_h, long long s_t,
    int BH, int Hkv, int n, int nseg, int seg_len, float* __restrict__ seg_tot, int first_tensor)
{
    __shared__ float part[16][kHeadDim];
    const int seg = blockIdx.x % (nseg - 1);
    const int chain = blockIdx.x / (nseg - 1);
    const int tensor = chain / BH + first_tensor, bh = chain % BH;
    const T* X = (tensor ? V : K) + (long long)(bh / Hkv) * s_b + (long long)(bh % Hkv) * s_h;
    const int l = threadIdx.x & 15, rg = threadIdx.x >> 4;
    const int t_begin = seg * seg_len;
    const int t_end = min(n, t_begin + seg_len);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int t0 = t_begin; t0 < t_end; t0 += kTile) {
        Row8<T> rows[kR];
        load_tile<false>(rows, X, s_t, t0 + rg * kR, t_end, 8 * l);
        if (t0 + kTile > t_end) clear_rows_past(rows, t0 + rg * kR, t_end);
#pragma unroll
        for (int r = 0; r < kR; ++r) {
            float x[8];
            rows[r].unpack(x);
#pragma unroll
            for (int c = 0; c < 8; ++c) acc[c] += x[c];
        }
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) part[rg][8 * l + c] = acc[c];
    __syncthreads();
    if (threadIdx.x < kHeadDim) {
        float s = 0.f;
#pragma unroll
        for (int g = 0; g < 16; ++g) s += part[g][threadIdx.x];
        seg_tot[((long long)chain * nseg + seg) * kHeadDim + threadIdx.x] = s;
    }
}

// EMA = false: the anchor is the exact mean of the rows before (Algorithm 1); EMA = true: the
// incremental anchor of Eq. 1, A <- gamma A + (1 - gamma) x from zero, each row scored against
// the anchor before it is folded in.  The same three phases carry a decay: a row group's total
// is weighted towards its end, prefixes are multiplied by gamma^8 per row group and gamma^32 per
// wave on their way, and a segment that does not start a chain is preceded by `warm` rows that
// are only folded into the anchor (gamma^warm is below 1e-10, so what lies further back has
// no weight left); no totals pass is needed.
// first_tensor: 0 to walk K and V, or, with a single tensor (key-only / value-only scores),
// the tensor to walk (0 = K, 1 = V).
// STREAM: see load_tile (chosen by the host from the size of K and V).
template <typename T, bool EMA, bool INCL, bool STREAM>
__global__ __launch_bounds__(kThreads) void scan_score_kernel(
    const T* __restrict__ K, const T* __restrict__ V, long long s_b, long long s_h, long long s_t,
    int BH, int Hkv, int n, int nseg, int seg_len, const float* __restrict__ seg_tot,
    float* __restrict__ sim_k, float* __restrict__ sim_v, int first_tensor, float gamma, int warm)
{
    __shared__ float wtot[2][4][kHeadDim];

    const int seg = blockIdx.x % nseg;
    const int chain = blockIdx.x / nseg;
    const int tensor = chain / BH + first_tensor, bh = chain % BH;
    const T* X = (tensor ? V : K) + (long long)(bh / Hkv) * s_b + (long long)(bh % Hkv) * s_h;
    float* sim = (tensor ? sim_v : sim_k) + (long long)bh * n;

    const int tid = threadIdx.x;
    const int l = tid & 15;          // column slice: columns 8l .. 8l+7
    const int rg = tid >> 4;         // row group in the tile: rows 8rg .. 8rg+7
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rgw = (tid >> 4) & 3;  // row group inside the wave

    const int t_out = seg * seg_len;  // first row this workgroup writes a score for
    const int t_begin = EMA ? max(0, t_out - warm) : t_out;
    const int t_end = min(n, t_out + seg_len);
    // decay factors of the incremental anchor
    const float g1 = gamma, w1 = 1.0f - gamma;
    const float g2 = g1 * g1, g4 = g2 * g2, g8 = g4 * g4, g16 = g8 * g8, g32 = g16 * g16;
    const float g_rgw = rgw == 0 ? 1.0f : (rgw == 1 ? g8 : (rgw == 2 ? g16 : g16 * g8));

    float carry[8];
#pragma unroll
    for (int c = 0; c < 8; ++c) carry[c] = 0.f;
    for (int s = 0; !EMA && s < seg; ++s) {
        const float* p = seg_tot + ((long long)chain * nseg + s) * kHeadDim + 8 * l;
        const float4 a = *reinterpret_cast<const float4*>(p);
        const float4 b = *reinterpret_cast<const float4*>(p + 4);
        carry[0] += a.x; carry[1] += a.y; carry[2] += a.z; carry[3] += a.w;
        carry[4] += b.x; carry[5] += b.y; carry[6] += b.z; carry[7] += b.w;
    }

    Row8<T> buf0[kR], buf1[kR], buf2[kR];
    load_tile<STREAM>(buf0, X, s_t, t_begin + rg * kR, t_end, 8 * l);
    load_tile<STREAM>(buf1, X, s_t, t_begin + kTile + rg * kR, t_end, 8 * l);

    int parity = 0;
    auto process = [&](Row8<T>* rows, int t0, bool first_tile) {
        float x[kR][8];
        float tot[8];
        if (t0 + kTile > t_end) clear_rows_past(rows, t0 + rg * kR, t_end);  // uniform branch
#pragma unroll
        for (int r = 0; r < kR; ++r) rows[r].unpack(x[r]);
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float s = x[0][c];
#pragma unroll
            for (int r = 1; r < kR; ++r) s = EMA ? fmaf(g1, s, x[r][c]) : s + x[r][c];
            tot[c] = EMA ? w1 * s : s;  // EMA: what these 8 rows add to the anchor after them
        }
        // exclusive scan of the row-group totals inside the wave (4 row groups of 16 lanes);
        // EMA: as seen at the start of this thread's row group
        float excl[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            float a = __shfl_up(tot[c], 16);
            a = rgw >= 1 ? a : 0.f;
            const float pair = EMA ? fmaf(g8, a, tot[c]) : tot[c] + a;
            float b = __shfl_up(pair, 32);
            b = rgw >= 2 ? b : 0.f;
            excl[c] = EMA ? fmaf(g8, b, a) : a + b;
        }
        if (rgw == 3) {
            float4* dst = reinterpret_cast<float4*>(&wtot[parity][wave][8 * l]);
            float wt[8];
#pragma unroll
            for (int c = 0; c < 8; ++c) wt[c] = EMA ? fmaf(g8, excl[c], tot[c]) : excl[c] + tot[c];
            dst[0] = make_float4(wt[0], wt[1], wt[2], wt[3]);
            dst[1] = make_float4(wt[4], wt[5], wt[6], wt[7]);
        }
        __syncthreads();
        float A[8], all[8];
#pragma unroll
        for (int c = 0; c < 8; ++c) { A[c] = 0.f; all[c] = carry[c]; }  // `all` runs on from the carry
        // (`wave` is uniform: what is "before this wave" is decided by scalar branches; written
        // as a per-lane condition it became 32 selects a tile)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float4* src = reinterpret_cast<const float4*>(&wtot[parity][w][8 * l]);
            const float4 a = src[0], b = src[1];
            const float v[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
            if (w == wave) {
#pragma unroll
                for (int c = 0; c < 8; ++c) A[c] = all[c];   // the waves before this one
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) all[c] = EMA ? fmaf(g32, all[c], v[c]) : all[c] + v[c];
        }
#pragma unroll
        for (int c = 0; c < 8; ++c) {
            carry[c] = all[c];
            A[c] = EMA ? fmaf(g_rgw, A[c], excl[c]) : A[c] + excl[c];
        }
        parity ^= 1;

        // replay the 8 rows against the running prefix; lane r of the DPP row keeps row r.
        // |A|^2 is taken directly for the thread's first row and then advanced with
        // |A + x|^2 = |A|^2 + 2 <A, x> + |x|^2 (EMA: |g A + w x|^2 = g^2 |A|^2 + 2 g w <A, x>
        // + w^2 |x|^2) from the two reductions that are needed anyway.  The chain's first tile
        // takes it directly for every row: there the prefix is a sum of few rows and may cancel.
        float my_dot = 0.f, my_aa = 0.f, my_xx = 0.f;
        float aa_run = 0.f;
#pragma unroll
        for (int r = 0; r < kR; ++r) {
            float dot = 0.f;
#pragma unroll
            for (int c = 0; c < 8; ++c) dot = fmaf(A[c], x[r][c], dot);
            if (r == 0 || first_tile) {
                float aa = 0.f;
#pragma unroll
                for (int c = 0; c < 8; ++c) aa = fmaf(A[c], A[c], aa);
                aa_run = row16_sum(aa);
            }
#pragma unroll
            for (int c = 0; c < 8; ++c) A[c] = EMA ? fmaf(g1, A[c], w1 * x[r][c]) : A[c] + x[r][c];
            dot = row16_sum(dot);
            const float xx = row16_sum(rows[r].sumsq());
            if (l == r) { my_dot = dot; my_aa = aa_run; my_xx = xx; }
            aa_run = EMA ? fmaf(g2, aa_run, fmaf(2.f * g1 * w1, dot, w1 * w1 * xx))
                         : fmaf(2.f, dot, aa_run + xx);
        }
        if (l < kR) {
            const int t = t0 + rg * kR + l;
            if (t < t_end && t >= t_out) {
                // cosine of row t with the MEAN of rows 0..t-1: numerator and denominator
                // both carry the 1/t so that the 1e-8 floor applies to |mean| * |x|
                // (the incremental anchor is carried as it is and needs no factor)
                // (INCL: against the anchor with row t already absorbed, whose product with
                // the row and whose norm follow from the same three reductions)
                float num = my_dot, aa = my_aa;
                int rows_in = t;
                if (INCL) {
                    if (EMA) {
                        num = fmaf(g1, my_dot, w1 * my_xx);
                        aa = fmaf(g2, my_aa, fmaf(2.f * g1 * w1, my_dot, w1 * w1 * my_xx));
                    } else {
                        num = my_dot + my_xx;
                        aa = fmaf(2.f, my_dot, my_aa + my_xx);
                        rows_in = t + 1;
                    }
                    aa = fmaxf(aa, 0.f);
                }
                const float inv_t = EMA ? 1.0f : (rows_in > 0 ? 1.0f / (float)rows_in : 0.f);
                const float den = fmaxf(sqrtf(aa) * sqrtf(my_xx) * inv_t, 1e-8f);
                float cs = (num * inv_t) / den;
                cs = fminf(1.f, fmaxf(-1.f, cs));
                store_score(sim + t, cs);
            }
        }
    };

    // two tiles in flight while a third is processed (rows past the end load as zeros)
    for (int t0 = t_begin; t0 < t_end; t0 += 3 * kTile) {
        load_tile<STREAM>(buf2, X, s_t, t0 + 2 * kTile + rg * kR, t_end, 8 * l);
        process(buf0, t0, t0 == 0);
        if (t0 + kTile >= t_end) break;
        load_tile<STREAM>(buf0, X, s_t, t0 + 3 * kTile + rg * kR, t_end, 8 * l);
        process(buf1, t0 + kTile, false);
        if (t0 + 2 * kTile >= t_end) break;
        load_tile<STREAM>(buf1, X, s_t, t0 + 4 * kTile + rg * kR, t_end, 8 * l);
        process(buf2, t0 + 2 * kTile, false);
    }
}

}  // namespace

ScorePlan plan_score(int B, int Hkv, int n)
{
    const int chains = 2 * B * Hkv;
    const int tiles = (n + kTile - 1) / kTile;
    int want = chains >= 256 ? 1 : (512 + chains - 1) / chains;
    int nseg = want < tiles ? want : tiles;
    if (nseg < 1) nseg = 1;
    const int tiles_per_seg = (tiles + nseg - 1) / nseg;
    nseg = (tiles + tiles_per_seg - 1) / tiles_per_seg;
    return ScorePlan{nseg, tiles_per_seg * kTile};
}

size_t score_scratch_floats(const Dims& d)
{
    const ScorePlan p = plan_score(d.B, d.Hkv, d.n);
    return (size_t)2 * d.B * d.Hkv * p.nseg * kHeadDim;
}

// Rows of warm-up before a segment of the incremental anchor: gamma^rows <= 1e-10, in whole
// tiles of the largest workgroup; 0 if no such count fits an int (gamma too close to one).
static int ema_warm_rows(float gamma)
{
    if (!(gamma > 0.f)) return kTile;
    const double rows = ceil(log(1e-10) / log((double)gamma));
    if (!(rows < 1e8)) return 0;
    return (int)((((long long)rows + kTile - 1) / kTile) * kTile);
}

template <typename T, bool EMA, bool INCL, typename... Args>
static void launch_scan(bool stream_loads, int grid, hipStream_t s, Args... args)
{
    if (stream_loads)
        scan_score_kernel<T, EMA, INCL, true><<<dim3(grid), dim3(kThreads), 0, s>>>(args...);
    else
        scan_score_kernel<T, EMA, INCL, false><<<dim3(grid), dim3(kThreads), 0, s>>>(args...);
}

template <typename T>
static hipError_t launch_score_t(const Dims& d, const T* K, const T* V, float* sim_k,
                                 float* sim_v, float* seg_tot, int tensors, int anchor,
                                 float gamma, hipStream_t s)
{
    ScorePlan p = plan_score(d.B, d.Hkv, d.n);
    const int BH = d.B * d.Hkv;
    const int n_tensors = tensors == 0 ? 2 : 1;
    const int first_tensor = tensors == 2 ? 1 : 0;
    const int chains = n_tensors * BH;
    const int inclusive = anchor >> 1;  // bit 1 of `anchor`: the anchor of a row includes the row
    anchor &= 1;
    // Tensors that together exceed the last-level cache (256 MB Infinity Cache) are streamed past
    // the L2: measured on whole steps, workload 2 (537 MB) -2.6 %, workload 3 (336 MB) -1.2 %;
    // below that size the later kernels find the rows in the caches and streaming costs
    // (workload 4, 67 MB: +0.7 %; workload 1, 17 MB: +12 %).
    const bool stream_loads = (double)chains * d.n * kHeadDim * sizeof(T) > 256.0 * 1024 * 1024;
    if (anchor == 1) {
        // segments only if their warm-up is at most as long as they are
        const int warm = ema_warm_rows(gamma);
        if (p.nseg > 1 && (warm == 0 || warm > p.seg_len)) {
            const int want = warm == 0 ? 1 : std::max(1, d.n / warm);
            const int tiles = (d.n + kTile - 1) / kTile;
            const int nseg = std::max(1, std::min(want, p.nseg));
            const int tiles_per_seg = (tiles + nseg - 1) / nseg;
            p = ScorePlan{(tiles + tiles_per_seg - 1) / tiles_per_seg, tiles_per_seg * kTile};
        }
        if (inclusive)
            launch_scan<T, true, true>(stream_loads, chains * p.nseg, s, K, V, d.kvs[0], d.kvs[1], d.kvs[2],
                                       BH, d.Hkv, d.n, p.nseg, p.seg_len, seg_tot, sim_k, sim_v,
                                       first_tensor, gamma, warm);
        else
            launch_scan<T, true, false>(stream_loads, chains * p.nseg, s, K, V, d.kvs[0], d.kvs[1], d.kvs[2],
                                        BH, d.Hkv, d.n, p.nseg, p.seg_len, seg_tot, sim_k, sim_v,
                                        first_tensor, gamma, warm);
        return hipGetLastError();
    }
    if (p.nseg > 1) {
        segment_totals_kernel<T><<<dim3(chains * (p.nseg - 1)), dim3(kThreads), 0, s>>>(
            K, V, d.kvs[0], d.kvs[1], d.kvs[2], BH, d.Hkv, d.n, p.nseg, p.seg_len, seg_tot,
            first_tensor);
    }
    if (inclusive)
        launch_scan<T, false, true>(stream_loads, chains * p.nseg, s, K, V, d.kvs[0], d.kvs[1], d.kvs[2], BH,
                                    d.Hkv, d.n, p.nseg, p.seg_len, seg_tot, sim_k, sim_v, first_tensor,
                                    0.f, 0);
    else
        launch_scan<T, false, false>(stream_loads, chains * p.nseg, s, K, V, d.kvs[0], d.kvs[1], d.kvs[2], BH,
                                     d.Hkv, d.n, p.nseg, p.seg_len, seg_tot, sim_k, sim_v, first_tensor,
                                     0.f, 0);
    return hipGetLastError();
}

hipError_t launch_score(const Dims& d, int dtype, const void* K, const void* V, float* sim_k,
                        float* sim_v, float* seg_tot, int tensors, int anchor, float gamma,
                        hipStream_t s)
{
    if (dtype == 0)
        return launch_score_t<float>(d, (const float*)K, (const float*)V, sim_k, sim_v, seg_tot,
                                     tensors, anchor, gamma, s);
    return launch_score_t<uint16_t>(d, (const uint16_t*)K, (const uint16_t*)V, sim_k, sim_v,
                                    seg_tot, tensors, anchor, gamma, s);
}

}  // namespace tf
