// Two measurement probes that put an on-box ceiling next to the vendor peaks the roofline
// fractions are quoted against: a plain streaming read of HBM and back-to-back bf16 MFMAs.
// They are not part of the token-filtering path.
#include "tf_kernels.h"

namespace tf {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Every thread reads 16-byte chunks with a grid stride and folds them into one word; the
// result is written only if it has a value no input produces, so the loads cannot be dropped.
__global__ __launch_bounds__(256) void stream_read_kernel(const uint4* __restrict__ src,
                                                          long long chunks, unsigned* sink)
{
    const long long stride = (long long)gridDim.x * blockDim.x;
    long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    unsigned acc = 0;
    for (; i + 3 * stride < chunks; i += 4 * stride) {
        const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], e = src[i + 3 * stride];
        acc ^= (a.x ^ a.y ^ a.z ^ a.w) ^ (b.x ^ b.y ^ b.z ^ b.w) ^ (c.x ^ c.y ^ c.z ^ c.w) ^
               (e.x ^ e.y ^ e.z ^ e.w);
    }
    for (; i < chunks; i += stride) {
        const uint4 a = src[i];
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u) *sink = acc;
}

// Four independent accumulator chains of v_mfma_f32_32x32x16_bf16 per wave, two waves per
// SIMD: nothing but the matrix pipe is busy.
__global__ __launch_bounds__(512) void mfma_chain_kernel(int iters, float seed, float* sink)
{
    bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(seed + threadIdx.x * 0.001f + i);
        b[i] = (__bf16)(seed - i);
    }
    f32x16 c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int it = 0; it < iters; ++it) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
    if (s == 12345.678f) *sink = s;
}

}  // namespace

hipError_t launch_probe_stream_read(const void* src, size_t bytes, void* sink, int n_cu,
                                    hipStream_t s)
{
    const long long chunks = (long long)(bytes / 16);
    stream_read_kernel<<<dim3(n_cu * 16), dim3(256), 0, s>>>((const uint4*)src, chunks,
                                                            (unsigned*)sink);
    return hipGetLastError();
}

// flops issued: grid * 8 waves * iters * 4 MFMAs * (2 * 32 * 32 * 16)
hipError_t launch_probe_mfma(int iters, void* sink, int n_cu, hipStream_t s)
{
    mfma_chain_kernel<<<dim3(n_cu), dim3(512), 0, s>>>(iters, 0.5f, (float*)sink);
    return hipGetLastError();
}

}  // namespace tf
