// Internal declarations shared by the HIP sources of the token-filter library (gfx950 only).
// Host launchers are declared here and defined next to their kernels; tokfilt_api.hip
// validates arguments and sequences them.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tf {

constexpr int kHeadDim = 128;

// Problem extents and element strides, passed by value to kernels.
struct Dims {
    int B, Hq, Hkv, n, m;
    long long qs[3];   // Q strides for (batch, head, position)
    long long kvs[3];  // K / V strides
    long long os[3];   // O strides
};

// ---- scoring: exclusive prefix sums of K and V along the sequence + per-head cosines -----
struct ScorePlan {
    int nseg;     // sequence segments per (tensor, batch, head) chain
    int seg_len;  // tokens per segment, a multiple of the scan tile
};
ScorePlan plan_score(int B, int Hkv, int n);
size_t score_scratch_floats(const Dims& d);  // segment totals
// sim_k / sim_v: [B][Hkv][n] float.  seg_tot: scratch of score_scratch_floats() floats.
// tensors: 0 = K and V, 1 = K only, 2 = V only.  anchor: bit 0: 0 = exact mean, 1 = incremental
// anchor with smoothing factor gamma; bit 1: the anchor of a row includes that row.
hipError_t launch_score(const Dims& d, int dtype, const void* K, const void* V, float* sim_k,
                        float* sim_v, float* seg_tot, int tensors, int anchor, float gamma,
                        hipStream_t s);

// ---- head statistics + variance-aware fusion ----------------------------------------------
hipError_t launch_fuse(const Dims& d, int fusion, const float* sim_k, const float* sim_v,
                       float* fused, hipStream_t s);

// ---- exact-count decision and stream compaction -------------------------------------------
hipError_t launch_select(const Dims& d, int warmup, const float* fused, uint8_t* keep,
                         float* tau, hipStream_t s);
hipError_t launch_compact(const Dims& d, const uint8_t* keep, int32_t* kept_idx, hipStream_t s);
// decision and compaction in one launch (rows of up to 32768 tokens; longer rows take the two
// kernels above)
hipError_t launch_select_compact(const Dims& d, int warmup, const float* fused, uint8_t* keep,
                                 int32_t* kept_idx, float* tau, hipStream_t s);
// online decision with an adaptive threshold: keep [B][n], kept_idx [B][n] (kept positions
// ascending, then -1), count [B], tau [B] (may be null)
hipError_t launch_select_online(const Dims& d, int warmup, float target, float eta, float tau0,
                                const float* fused, uint8_t* keep, int32_t* kept_idx,
                                int32_t* count, float* tau, hipStream_t s);
// every token kept: keep = 1, kept_idx = 0 .. n-1, tau = +inf (tau may be null)
hipError_t launch_keep_all(const Dims& d, uint8_t* keep, int32_t* kept_idx, float* tau,
                           hipStream_t s);
// no token kept: keep = 0, tau = -inf (tau may be null)
hipError_t launch_keep_none(const Dims& d, uint8_t* keep, float* tau, hipStream_t s);
// keep mask from an index list (for callers that bring their own kept set)
hipError_t launch_mask_from_idx(const Dims& d, const int32_t* kept_idx, uint8_t* keep,
                                const int32_t* counts, long long idx_stride, hipStream_t s);

// ---- attention over the kept tokens -------------------------------------------------------
hipError_t launch_zero_filtered(const Dims& d, int dtype, const uint8_t* keep, void* O,
                                hipStream_t s);
// counts (may be null): per-row numbers of kept tokens [B]; kept_idx rows are then idx_stride
// apart and d.m is only the bound on a row's count
hipError_t launch_attend_f32(const Dims& d, float scale, const float* Q, const float* K,
                             const float* V, const int32_t* kept_idx, float* O,
                             const int32_t* counts, long long idx_stride, hipStream_t s);
// also writes the zero rows of filtered positions (kept_idx strictly ascending).  n_cu: compute
// units of the device (one persistent workgroup each); n_xcd: its accelerator dies (each with an
// L2 of its own).  hipErrorInvalidValue if a (batch, head) slice of K / V spans 4 GiB or more.
hipError_t launch_attend_bf16(const Dims& d, float scale, const void* Q, const void* K,
                              const void* V, const int32_t* kept_idx, void* O, int n_cu, int n_xcd,
                              const int32_t* counts, long long idx_stride, hipStream_t s);

// ---- per-token (decoding) form ----------------------------------------------------------------
constexpr int kDecodeMaxSplit = 16;                 // slices of a row's cache per query head
constexpr int kDecodePartFloats = kHeadDim + 2;     // floats of one slice's partial result
struct DecodeArgs {
    int B, Hq, Hkv, capacity;
    double *anchor_k, *anchor_v;                    // [B][Hkv][128]
    int32_t *seen, *skipped, *cache_len, *overflow; // [B]
    float* tau;                                     // [B]
    void *k_cache, *v_cache;                        // [B][Hkv][capacity][128]
    int ema, inclusive, fusion, warmup;
    double gamma;
    float target, eta, scale;
    uint8_t* skip;                                  // out [B]
    float* fused;                                   // out [B]
    float* part;                                    // scratch [B][Hq][n_split][kDecodePartFloats]
    int n_split;                                    // 1 .. kDecodeMaxSplit
};
hipError_t launch_decode_init(const DecodeArgs& a, float tau0, hipStream_t s);
// state after a prompt of n rows that the batched online path has processed: anchors from K and
// V (element strides kvs for batch, head, position), caches from the kept rows (kept_idx
// [B][n], count [B]), counters; the threshold is written by the decision kernel itself
hipError_t launch_decode_seed(const DecodeArgs& a, int dtype, const void* K, const void* V,
                              const int32_t* kept_idx, const int32_t* count, int n,
                              const long long* kvs, hipStream_t s);
// q, o: [B][Hq][128]; k, v: [B][Hkv][128]
hipError_t launch_decode_step(const DecodeArgs& a, int dtype, const void* q, const void* k,
                              const void* v, void* o, hipStream_t s);

// ---- measurement probes (not part of the path) ---------------------------------------------
hipError_t launch_probe_stream_read(const void* src, size_t bytes, void* sink, int n_cu,
                                    hipStream_t s);
hipError_t launch_probe_mfma(int iters, void* sink, int n_cu, hipStream_t s);

// ---- small device helpers -----------------------------------------------------------------
#ifdef __HIPCC__
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// Sum over each aligned group of 16 lanes (one DPP row); every lane ends with the total.
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);  // row_half_mirror
    v += dpp_mov<0x140>(v);  // row_mirror
    return v;
}

// The gfx950 half swaps, on floats.  With a = (a0 a1 a2 a3) and b = (b0 b1 b2 b3) in 16-lane
// rows: swap16 returns first = (a0 b0 a2 b2), second = (a1 b1 a3 b3); swap32 returns
// first = (a0 a1 b0 b1), second = (a2 a3 b2 b3).  Both results go through an opaque move before
// they are reinterpreted as floats: this compiler's bit cast of the second result silently
// picks up the first one.
struct FloatPair { float first, second; };
__device__ __forceinline__ FloatPair swap16(float a, float b)
{
    const auto r = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, a),
                                                    __builtin_bit_cast(unsigned, b), false, false);
    unsigned r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    return FloatPair{__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1)};
}
__device__ __forceinline__ FloatPair swap32(float a, float b)
{
    const auto r = __builtin_amdgcn_permlane32_swap(__builtin_bit_cast(unsigned, a),
                                                    __builtin_bit_cast(unsigned, b), false, false);
    unsigned r0 = r[0], r1 = r[1];
    asm volatile("" : "+v"(r0), "+v"(r1));
    return FloatPair{__builtin_bit_cast(float, r0), __builtin_bit_cast(float, r1)};
}
#endif

}  // namespace tf
