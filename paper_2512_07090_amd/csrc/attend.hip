// Causal softmax attention over the kept tokens (Section 3.2: filtered tokens get a zero
// attention output; the rest attend as usual, here to kept tokens only).  Queries and keys are
// addressed through kept_idx, so "causal" is "key rank <= query rank" in the compacted order.
//
//   zero_filtered_kernel  writes the zero rows of O for filtered positions;
//   attend_f32_kernel     plain fp32 tiles (the fp32 correctness configuration);
//   attend_bf16_kernel    flash-style, bf16 MFMA 32x32x16 with fp32 accumulation and online
//                         softmax; K tiles and transposed V tiles staged in LDS.
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
                                                         float* __restrict__ O)
{
    __shared__ float Qs[kFM][kFStride];
    __shared__ float Ks[kFN][kFStride];
    __shared__ float Vs[kFN][kHeadDim];
    __shared__ float Ps[kFM][kFN + 1];

    const int qt = blockIdx.x, hq = blockIdx.y, b = blockIdx.z;
    const int hk = hq / (d.Hq / d.Hkv);
    const int32_t* idx = kept_idx + (long long)b * d.m;
    const float* Qb = Q + (long long)b * d.qs[0] + (long long)hq * d.qs[1];
    const float* Kb = K + (long long)b * d.kvs[0] + (long long)hk * d.kvs[1];
    const float* Vb = V + (long long)b * d.kvs[0] + (long long)hk * d.kvs[1];
    const int tid = threadIdx.x;
    const int row = tid >> 3, g = tid & 7;  // tile row handled when loading / computing
    const int i0 = qt * kFM;
    const int i = i0 + row;                 // this thread's query rank

    {
        const bool ok = i < d.m;
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
            const bool ok = j < d.m;
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
            s[kk] = (j <= i && j < d.m) ? s[kk] * scale : -1e30f;
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
    if (i < d.m) {
        float* dst = O + (long long)b * d.os[0] + (long long)hq * d.os[1] + (long long)idx[i] * d.os[2];
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4)
            *reinterpret_cast<float4*>(dst + 4 * g + 32 * q4) =
                make_float4(o[4 * q4] * inv, o[4 * q4 + 1] * inv, o[4 * q4 + 2] * inv, o[4 * q4 + 3] * inv);
    }
}

// ------------------------------------------------------------------------------ bf16 MFMA path
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBM = 128;                  // kept queries per workgroup (32 per wave)
constexpr int kBN = 64;                   // kept keys per tile
constexpr int kKStr = kHeadDim + 8;       // K tile row stride in elements (272 B)
constexpr int kVStr = kBN + 4;            // transposed V tile row stride in elements (136 B)
constexpr int kKTile = kBN * kKStr;       // elements
constexpr int kVTile = kHeadDim * kVStr;  // elements

// Register image of one K/V tile in flight from global memory to LDS.
struct TileRegs {
    uint4 k[4];      // 4 x 16 B of K rows
    unsigned v[16];  // 4 units x 4 keys x (2 adjacent d) of V
};

__device__ __forceinline__ void tile_load(TileRegs& r, const uint16_t* __restrict__ Kb,
                                          const uint16_t* __restrict__ Vb, long long s_t,
                                          const int32_t* __restrict__ idx, int j0, int m, int tid)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i;
        const int row = c >> 4, col = (c & 15) * 8;
        const int j = j0 + row;
        if (j < m)
            r.k[i] = *reinterpret_cast<const uint4*>(Kb + (long long)idx[j] * s_t + col);
        else
            r.k[i] = make_uint4(0, 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int u = tid + 256 * i;
        const int dp = u & 63, kq = u >> 6;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const int j = j0 + 4 * kq + kk;
            r.v[4 * i + kk] = j < m ? *reinterpret_cast<const unsigned*>(
                                          Vb + (long long)idx[j] * s_t + 2 * dp)
                                    : 0u;
        }
    }
}

__device__ __forceinline__ void tile_store(const TileRegs& r, uint16_t* Ks, uint16_t* Vt, int tid)
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int c = tid + 256 * i;
        const int row = c >> 4, col = (c & 15) * 8;
        *reinterpret_cast<uint4*>(Ks + row * kKStr + col) = r.k[i];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int u = tid + 256 * i;
        const int dp = u & 63, kq = u >> 6;
        const unsigned a = r.v[4 * i], b = r.v[4 * i + 1], c = r.v[4 * i + 2], e = r.v[4 * i + 3];
        // even d: low halves of the four keys; odd d: high halves
        uint2 even, odd;
        even.x = __builtin_amdgcn_perm(b, a, 0x05040100u);
        even.y = __builtin_amdgcn_perm(e, c, 0x05040100u);
        odd.x = __builtin_amdgcn_perm(b, a, 0x07060302u);
        odd.y = __builtin_amdgcn_perm(e, c, 0x07060302u);
        *reinterpret_cast<uint2*>(Vt + (2 * dp) * kVStr + 4 * kq) = even;
        *reinterpret_cast<uint2*>(Vt + (2 * dp + 1) * kVStr + 4 * kq) = odd;
    }
}

__global__ __launch_bounds__(256, 2) void attend_bf16_kernel(Dims d, float scale_log2, int n_qt,
                                                             int total_blocks,
                                                             const uint16_t* __restrict__ Q,
                                                             const uint16_t* __restrict__ K,
                                                             const uint16_t* __restrict__ V,
                                                             const int32_t* __restrict__ kept_idx,
                                                             uint16_t* __restrict__ O)
{
    __shared__ __attribute__((aligned(16))) uint16_t Ks[2][kKTile];
    __shared__ __attribute__((aligned(16))) uint16_t Vt[2][kVTile];

    // Workgroup ids are dealt round-robin to the 8 XCDs; renumber so that each XCD gets a
    // contiguous run of (batch, head) groups (its L2 then holds that group's K and V), and
    // inside a group start with the last, longest query tile.
    const int per_xcd = total_blocks >> 3;
    const int logical = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    const int bh = logical / n_qt;
    if (bh >= d.B * d.Hq) return;
    const int qt = n_qt - 1 - logical % n_qt;
    const int b = bh / d.Hq, hq = bh % d.Hq;
    const int hk = hq / (d.Hq / d.Hkv);

    const int32_t* idx = kept_idx + (long long)b * d.m;
    const uint16_t* Qb = Q + (long long)b * d.qs[0] + (long long)hq * d.qs[1];
    const uint16_t* Kb = K + (long long)b * d.kvs[0] + (long long)hk * d.kvs[1];
    const uint16_t* Vb = V + (long long)b * d.kvs[0] + (long long)hk * d.kvs[1];
    uint16_t* Ob = O + (long long)b * d.os[0] + (long long)hq * d.os[1];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hh = lane >> 5;

    const int i0 = qt * kBM;
    const int iw = i0 + 32 * wave;   // first query rank of this wave
    const int iq = iw + col;         // this lane's query rank
    const int i_last = min(i0 + kBM, d.m) - 1;
    const int n_kt = i_last / kBN + 1;

    // Q fragments (B operand of S^T = K Q^T): lane (col, hh) holds, for k-step s, the 8
    // elements d = 16 s + 8 hh .. +7 of query row `col`.
    bf16x8 qf[8];
    {
        const bool ok = iq < d.m;
        const uint16_t* src = Qb + (ok ? (long long)idx[iq] * d.qs[2] : 0);
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            uint4 raw = make_uint4(0, 0, 0, 0);
            if (ok) raw = *reinterpret_cast<const uint4*>(src + 16 * s + 8 * hh);
            qf[s] = __builtin_bit_cast(bf16x8, raw);
        }
    }

    f32x16 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
    float m_run = -1e30f, l_run = 0.f;

    TileRegs regs;
    tile_load(regs, Kb, Vb, d.kvs[2], idx, 0, d.m, tid);
    tile_store(regs, Ks[0], Vt[0], tid);
    __syncthreads();

    for (int kt = 0; kt < n_kt; ++kt) {
        const int cur = kt & 1;
        const int j0 = kt * kBN;
        const bool more = kt + 1 < n_kt;
        if (more) tile_load(regs, Kb, Vb, d.kvs[2], idx, j0 + kBN, d.m, tid);

        if (j0 <= iw + 31) {
            const uint16_t* ks = Ks[cur];
            const uint16_t* vt = Vt[cur];
            // S^T (keys x queries): two 32-key subtiles
            f32x16 sacc[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[mt][v] = 0.f;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8*>(
                        ks + (32 * mt + col) * kKStr + 16 * s + 8 * hh);
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[mt], 0, 0, 0);
                }
            }
            // accumulator register v of subtile mt is key j0 + 32 mt + 8 (v / 4) + 4 hh + v % 4
            const bool diag = j0 + kBN - 1 > iw || j0 + kBN > d.m;
            float mx = -1e30f;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    float s = sacc[mt][v] * scale_log2;
                    if (diag) {
                        const int j = j0 + 32 * mt + 8 * (v >> 2) + 4 * hh + (v & 3);
                        if (j > iq || j >= d.m) s = -1e30f;
                    }
                    sacc[mt][v] = s;
                    mx = fmaxf(mx, s);
                }
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float m_new = fmaxf(m_run, mx);
            const float corr = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            float psum = 0.f;
            bf16x8 pf[4];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float s = sacc[mt][v];
                    const float p = s > -1e29f ? __builtin_amdgcn_exp2f(s - m_new) : 0.f;
                    psum += p;
                    pf[2 * mt + (v >> 3)][v & 7] = (__bf16)p;
                }
            l_run = l_run * corr + psum;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[dt][v] *= corr;
            // O^T (d x queries) += V^T P^T; k-slot e of k-step ks is key
            // 16 ks + 8 (e / 4) + 4 hh + e % 4 of the tile, for both operands
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
#pragma unroll
                for (int ks4 = 0; ks4 < 4; ++ks4) {
                    const uint16_t* vp = vt + (32 * dt + col) * kVStr + 16 * ks4 + 4 * hh;
                    const uint2 lo = *reinterpret_cast<const uint2*>(vp);
                    const uint2 hi = *reinterpret_cast<const uint2*>(vp + 8);
                    const uint4 raw = make_uint4(lo.x, lo.y, hi.x, hi.y);
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, raw), pf[ks4], oacc[dt], 0, 0, 0);
                }
            }
        }

        if (more) tile_store(regs, Ks[cur ^ 1], Vt[cur ^ 1], tid);
        __syncthreads();
    }

    // normalise, transpose through LDS (the K buffers are free now) and write whole rows
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    uint16_t* os = &Ks[0][0] + wave * (32 * kKStr);  // [32 queries][kKStr]
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
            bf16x4 o4;
#pragma unroll
            for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[dt][4 * v4 + e] * inv);
            *reinterpret_cast<bf16x4*>(os + col * kKStr + 32 * dt + 8 * v4 + 4 * hh) = o4;
        }
    __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): this wave's LDS writes have landed
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int it = 0; it < 8; ++it) {
        const int r = 4 * it + (lane >> 4);
        const int i = iw + r;
        if (i < d.m) {
            const uint4 v = *reinterpret_cast<const uint4*>(os + r * kKStr + 8 * (lane & 15));
            *reinterpret_cast<uint4*>(Ob + (long long)idx[i] * d.os[2] + 8 * (lane & 15)) = v;
        }
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
                             const float* V, const int32_t* kept_idx, float* O, hipStream_t s)
{
    dim3 grid((d.m + kFM - 1) / kFM, d.Hq, d.B);
    attend_f32_kernel<<<grid, dim3(256), 0, s>>>(d, scale, Q, K, V, kept_idx, O);
    return hipGetLastError();
}

hipError_t launch_attend_bf16(const Dims& d, float scale, const void* Q, const void* K,
                              const void* V, const int32_t* kept_idx, void* O, hipStream_t s)
{
    const int n_qt = (d.m + kBM - 1) / kBM;
    const int blocks = n_qt * d.Hq * d.B;
    const int total = (blocks + 7) & ~7;
    attend_bf16_kernel<<<dim3(total), dim3(256), 0, s>>>(
        d, scale * 1.44269504088896340736f, n_qt, total, (const uint16_t*)Q, (const uint16_t*)K,
        (const uint16_t*)V, kept_idx, (uint16_t*)O);
    return hipGetLastError();
}

}  // namespace tf
