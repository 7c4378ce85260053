// Causal softmax attention over the kept tokens (Section 3.2: filtered tokens get a zero
// attention output; the rest attend as usual, here to kept tokens only).  Queries and keys are
// addressed through kept_idx, so "causal" is "key rank <= query rank" in the compacted order.
//
//   zero_filtered_kernel  writes the zero rows of O for filtered positions;
//   attend_f32_kernel     plain fp32 tiles (the fp32 correctness configuration).
// The bf16 MFMA kernel lives in attend_bf16.hip.
#include "tf_kernels.h"

namespace tf {

namespace {

// ------------------------------------------------------------------------------ zero rows
// 16 lanes per row (16 B each for bf16, 32 B for fp32), 16 rows per workgroup.
template <int ELEM_BYTES>
__global__ __launch_bounds__(256) void zero_filtered_kernel(Dims d, const uint8_t* __restrict__ keep,
                                                            char* __restrict__ O)
{
    const int pos = blockIdx.x * 16 + (threadIdx.x >> 4);
    const int hq = blockIdx.y, b = blockIdx.z;
    if (pos >= d.n || keep[(long long)b * d.n + pos]) return;
    char* row = O + ((long long)b * d.os[0] + (long long)hq * d.os[1] + (long long)pos * d.os[2]) * ELEM_BYTES;
    const int l = threadIdx.x & 15;
    const uint4 z = make_uint4(0, 0, 0, 0);
    if (ELEM_BYTES == 2) {
        reinterpret_cast<uint4*>(row)[l] = z;
    } else {
        reinterpret_cast<uint4*>(row)[l] = z;
        reinterpret_cast<uint4*>(row)[16 + l] = z;
    }
}

// ------------------------------------------------------------------------------ fp32 path
constexpr int kFM = 32, kFN = 32, kFStride = kHeadDim + 4;

__global__ __launch_bounds__(256) void attend_f32_kernel(Dims d, float scale,
                                                         const float* __restrict__ Q,
                                                         const float* __restrict__ K,
                                                         const float* __restrict__ V,
                                                         const int32_t* __restrict__ kept_idx,
                                                         float* __restrict__ O,
                                                         const int32_t* __restrict__ counts,
                                                         long long idx_stride)
{
    __shared__ float Qs[kFM][kFStride];
    __shared__ float Ks[kFN][kFStride];
    __shared__ float Vs[kFN][kHeadDim];
    __shared__ float Ps[kFM][kFN + 1];

    const int qt = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int hk = hq / (d.Hq / d.Hkv);
    // kept tokens of this batch row (per row when counts is given: d.m is then the bound)
    const int m = counts ? counts[b] : d.m;
    if (blockIdx.x * kFM >= m) return;
    const int32_t* idx = kept_idx + (long long)b * idx_stride;
    const float* Qb = Q + (long long)b * d.qs[0] + (long long)hq * d.qs[1];
    const float* Kb = K + (long long)b * d.kvs[0] + (long long)hk * d.kvs[1];
    const float* Vb = V + (long long)b * d.kvs[0] + (long long)hk * d.kvs[1];
    const int tid = threadIdx.x;
    const int row = tid >> 3, g = tid & 7;  // tile row handled when loading / computing
    const int i0 = qt * kFM;
    const int i = i0 + row;                 // this thread's query rank

    {
        const bool ok = i < m;
        const float* src = ok ? Qb + (long long)idx[i] * d.qs[2] : Qb;
#pragma unroll
        for (int c4 = 0; c4 < 4; ++c4) {
            const int col = 4 * (g + 8 * c4);
            const float4 v = ok ? *reinterpret_cast<const float4*>(src + col) : make_float4(0, 0, 0, 0);
            *reinterpret_cast<float4*>(&Qs[row][col]) = v;
        }
    }

    float m_run = -1e30f, l_run = 0.f;
    float o[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) o[e] = 0.f;

    for (int kt = 0; kt <= qt; ++kt) {
        const int j0 = kt * kFN;
        __syncthreads();
        {
            const int j = j0 + row;
            const bool ok = j < m;
            const long long p = ok ? idx[j] : 0;
#pragma unroll
            for (int c4 = 0; c4 < 4; ++c4) {
                const int col = 4 * (g + 8 * c4);
                const float4 z = make_float4(0, 0, 0, 0);
                *reinterpret_cast<float4*>(&Ks[row][col]) =
                    ok ? *reinterpret_cast<const float4*>(Kb + p * d.kvs[2] + col) : z;
                *reinterpret_cast<float4*>(&Vs[row][col]) =
                    ok ? *reinterpret_cast<const float4*>(Vb + p * d.kvs[2] + col) : z;
            }
        }
        __syncthreads();

        // scores of query `row` against keys g, g+8, g+16, g+24 of the tile
        float s[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 8
        for (int c = 0; c < kHeadDim; ++c) {
            const float qv = Qs[row][c];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) s[kk] = fmaf(qv, Ks[g + 8 * kk][c], s[kk]);
        }
        float mx = -1e30f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int j = j0 + g + 8 * kk;
            s[kk] = (j <= i && j < m) ? s[kk] * scale : -1e30f;
            mx = fmaxf(mx, s[kk]);
        }
        mx = fmaxf(mx, __shfl_xor(mx, 1));
        mx = fmaxf(mx, __shfl_xor(mx, 2));
        mx = fmaxf(mx, __shfl_xor(mx, 4));
        const float m_new = fmaxf(m_run, mx);
        const float corr = expf(m_run - m_new);
        float psum = 0.f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const float p = s[kk] > -1e29f ? expf(s[kk] - m_new) : 0.f;
            Ps[row][g + 8 * kk] = p;
            psum += p;
        }
        psum += __shfl_xor(psum, 1);
        psum += __shfl_xor(psum, 2);
        psum += __shfl_xor(psum, 4);
        l_run = l_run * corr + psum;
        m_run = m_new;
#pragma unroll
        for (int e = 0; e < 16; ++e) o[e] *= corr;
        __syncthreads();
        // output columns 4g + 32q4 + (0..3), q4 = 0..3
        for (int k = 0; k < kFN; ++k) {
            const float p = Ps[row][k];
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const float4 v = *reinterpret_cast<const float4*>(&Vs[k][4 * g + 32 * q4]);
                o[4 * q4 + 0] = fmaf(p, v.x, o[4 * q4 + 0]);
                o[4 * q4 + 1] = fmaf(p, v.y, o[4 * q4 + 1]);
                o[4 * q4 + 2] = fmaf(p, v.z, o[4 * q4 + 2]);
                o[4 * q4 + 3] = fmaf(p, v.w, o[4 * q4 + 3]);
            }
        }
    }
    if (i < m) {
        float* dst = O + (long long)b * d.os[0] + (long long)hq * d.os[1] + (long long)idx[i] * d.os[2];
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
            *reinterpret_cast<float4*>(dst + 4 * g + 32 * q4) =
                make_float4(o[4 * q4] * inv, o[4 * q4 + 1] * inv, o[4 * q4 + 2] * inv, o[4 * q4 + 3] * inv);
    }
}

}  // namespace

hipError_t launch_zero_filtered(const Dims& d, int dtype, const uint8_t* keep, void* O,
                                hipStream_t s)
{
    dim3 grid((d.n + 15) / 16, d.Hq, d.B);
    if (dtype == 0)
        zero_filtered_kernel<4><<<grid, dim3(256), 0, s>>>(d, keep, (char*)O);
    else
        zero_filtered_kernel<2><<<grid, dim3(256), 0, s>>>(d, keep, (char*)O);
    return hipGetLastError();
}

hipError_t launch_attend_f32(const Dims& d, float scale, const float* Q, const float* K,
                             const float* V, const int32_t* kept_idx, float* O,
                             const int32_t* counts, long long idx_stride, hipStream_t s)
{
    dim3 grid((d.m + kFM - 1) / kFM, d.Hq, d.B);
    attend_f32_kernel<<<grid, dim3(256), 0, s>>>(d, scale, Q, K, V, kept_idx, O, counts,
                                                 counts ? idx_stride : (long long)d.m);
    return hipGetLastError();
}

}  // namespace tf
