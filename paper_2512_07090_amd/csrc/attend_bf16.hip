// Causal softmax attention over the kept tokens, bf16 inputs (Section 3.2: the tokens that
// are not skipped attend as usual; here both queries and keys are the kept tokens, addressed
// through kept_idx, so "causal" means key rank <= query rank in the compacted order).
//
// Flash-style kernel for gfx950.  One workgroup = NW waves x 32 kept queries; it walks the key
// tiles (64 kept keys) once, K and V rows gathered through kept_idx into LDS (row-major,
// double-buffered, the next tile's global loads in flight during the current tile's math).
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q fragments held in
//                 registers for the whole kernel.  The transposed product puts one query per
//                 lane column, so the online-softmax row statistics need a single cross-lane
//                 exchange (lane <-> lane + 32) per tile.
//   O^T += V^T P^T  A = V^T fragments read from the row-major V tile with the LDS transpose
//                 read (ds_read_b64_tr_b16), B = P^T converted to bf16 straight from the S^T
//                 accumulator registers.  The contraction order over keys is permuted the same
//                 way for both operands (accumulator register v of a 32-key block is key
//                 8 (v / 4) + 4 (lane / 32) + v % 4), which is free because a sum is taken.
//   softmax       fp32, base 2 (scale * log2 e folded into one FMA per score), running max
//                 only moved when it grows by more than 2^8 so the O rescale is rare.
#include "tf_kernels.h"

namespace tf {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short i16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kBN = 64;                  // kept keys per tile
constexpr int kKStr = kHeadDim + 8;      // K tile row stride, elements (272 B)
constexpr int kVStr = kHeadDim + 32;     // V tile row stride, elements (320 B)
constexpr int kKTile = kBN * kKStr;      // elements per K tile
constexpr int kVTile = kBN * kVStr;      // elements per V tile
constexpr int kStage = kKTile + kVTile;  // elements per pipeline stage
constexpr float kMaxSlack = 8.0f;        // running max may lag the true max by 2^8

template <int NW>
struct TileRegs {
    static constexpr int kChunks = 1024 / (64 * NW);  // 16-byte chunks per thread per tensor
    uint4 k[kChunks];
    uint4 v[kChunks];
};

// LDS transpose read: inside each group of 16 lanes, lane i receives element i % 4 of the
// four 8-byte rows addressed by lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12.
__device__ __forceinline__ i16x4 lds_read_tr16(const uint16_t* p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) i16x4*)(p));
}

template <int NW>
__global__ __launch_bounds__(64 * NW) void attend_bf16_kernel(
    Dims d, float scale_log2, int n_qt, int total_blocks, const uint16_t* __restrict__ Q,
    const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const int32_t* __restrict__ kept_idx, uint16_t* __restrict__ O)
{
    constexpr int NT = 64 * NW;
    constexpr int BM = 32 * NW;
    constexpr int CH = TileRegs<NW>::kChunks;
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kStage];

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
    const long long s_t = d.kvs[2];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, hh = lane >> 5;

    const int i0 = qt * BM;
    const int iw = i0 + 32 * wave;   // first query rank of this wave
    const int iq = iw + col;         // this lane's query rank
    const int i_last = min(i0 + BM, d.m) - 1;
    const int n_kt = i_last / kBN + 1;

    // tile-load roles: chunk c = tid + NT * i covers row c / 16, columns 8 (c % 16) ..+7
    int row_of[CH], col_of[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) {
        const int c = tid + NT * i;
        row_of[i] = c >> 4;
        col_of[i] = (c & 15) * 8;
    }

    auto load_idx = [&](int* pos, int j0) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            const int j = j0 + row_of[i];
            pos[i] = j < d.m ? idx[j] : -1;
        }
    };
    auto load_tile = [&](TileRegs<NW>& r, const int* pos) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            if (pos[i] >= 0) {
                const long long off = (long long)pos[i] * s_t + col_of[i];
                r.k[i] = *reinterpret_cast<const uint4*>(Kb + off);
                r.v[i] = *reinterpret_cast<const uint4*>(Vb + off);
            } else {
                r.k[i] = make_uint4(0, 0, 0, 0);
                r.v[i] = make_uint4(0, 0, 0, 0);
            }
        }
    };
    auto store_tile = [&](const TileRegs<NW>& r, uint16_t* stage) {
#pragma unroll
        for (int i = 0; i < CH; ++i) {
            *reinterpret_cast<uint4*>(stage + row_of[i] * kKStr + col_of[i]) = r.k[i];
            *reinterpret_cast<uint4*>(stage + kKTile + row_of[i] * kVStr + col_of[i]) = r.v[i];
        }
    };

    // Q fragments (B operand of S^T = K Q^T): lane (col, hh) holds, for k-step s, the 8
    // elements 16 s + 8 hh .. +7 of query row `col`.
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
    float m_run = -1e30f;  // running max of the RAW scores (may lag, see kMaxSlack)
    float l_run = 0.f;     // this lane's share of the softmax denominator

    TileRegs<NW> regs;
    int pos_a[CH], pos_b[CH];
    load_idx(pos_a, 0);
    load_tile(regs, pos_a);
    load_idx(pos_b, kBN);
    store_tile(regs, smem);
    __syncthreads();

    // LDS offsets of this lane's operand fragments inside a stage
    const int k_off = col * kKStr + 8 * hh;
    const int v_off = kKTile + (4 * hh + ((lane & 15) >> 2)) * kVStr + 16 * ((lane >> 4) & 1) +
                      4 * (lane & 3);

    for (int kt = 0; kt < n_kt; ++kt) {
        const int cur = kt & 1;
        const int j0 = kt * kBN;
        const bool more = kt + 1 < n_kt;
        if (more) {
            load_tile(regs, pos_b);
            load_idx(pos_b, j0 + 2 * kBN);
        }

        if (j0 <= iw + 31) {
            const uint16_t* st = smem + cur * kStage;
            // S^T (keys x queries): two 32-key blocks
            f32x16 sacc[2];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int v = 0; v < 16; ++v) sacc[mt][v] = 0.f;
#pragma unroll
                for (int s = 0; s < 8; ++s) {
                    const bf16x8 kf = *reinterpret_cast<const bf16x8*>(
                        st + k_off + 32 * mt * kKStr + 16 * s);
                    sacc[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc[mt], 0, 0, 0);
                }
            }
            // accumulator register v of block mt is key j0 + 32 mt + 8 (v / 4) + 4 hh + v % 4
            if (j0 + kBN - 1 > iw || j0 + kBN > d.m) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int j = j0 + 32 * mt + 8 * (v >> 2) + 4 * hh + (v & 3);
                        if (j > iq || j >= d.m) sacc[mt][v] = -1e30f;
                    }
            }
            float mx = fmaxf(sacc[0][0], sacc[1][0]);
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, fmaxf(sacc[0][v], sacc[1][v]));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            // move the running max only when the tile exceeds it by more than the slack
            const bool grow = mx > m_run + kMaxSlack;
            if (__any(grow)) {
                const float m_new = grow ? mx : m_run;
                const float corr = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);
                m_run = m_new;
                l_run *= corr;
#pragma unroll
                for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[dt][v] *= corr;
            }
            const float mc = m_run * scale_log2;
            float psum = 0.f;
            bf16x8 pf[4];
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float p = __builtin_amdgcn_exp2f(fmaf(sacc[mt][v], scale_log2, -mc));
                    psum += p;
                    pf[2 * mt + (v >> 3)][v & 7] = (__bf16)p;
                }
            l_run += psum;
            // O^T (d x queries) += V^T P^T.  k-slot e of k-step ks is key
            // 16 ks + 8 (e / 4) + 4 hh + e % 4 of the tile for both operands.
#pragma unroll
            for (int ks4 = 0; ks4 < 4; ++ks4) {
#pragma unroll
                for (int dt = 0; dt < 4; ++dt) {
                    const uint16_t* vp = st + v_off + 16 * ks4 * kVStr + 32 * dt;
                    const i16x4 lo = lds_read_tr16(vp);
                    const i16x4 hi = lds_read_tr16(vp + 8 * kVStr);
                    const i16x4 both[2] = {lo, hi};
                    oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, both), pf[ks4], oacc[dt], 0, 0, 0);
                }
            }
        }

        if (more) store_tile(regs, smem + (cur ^ 1) * kStage);
        __syncthreads();
    }

    // normalise, transpose through LDS (all tiles are consumed) and write whole rows
    const float l_tot = l_run + __shfl_xor(l_run, 32);
    const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
    uint16_t* os = smem + wave * (32 * kKStr);  // [32 queries][kKStr]
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v4 = 0; v4 < 4; ++v4) {
            bf16x4 o4;
#pragma unroll
            for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[dt][4 * v4 + e] * inv);
            *reinterpret_cast<bf16x4*>(os + col * kKStr + 32 * dt + 8 * v4 + 4 * hh) = o4;
        }
    __syncthreads();
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

hipError_t launch_attend_bf16(const Dims& d, float scale, const void* Q, const void* K,
                              const void* V, const int32_t* kept_idx, void* O, hipStream_t s)
{
    constexpr int NW = 8;
    constexpr int BM = 32 * NW;
    const int n_qt = (d.m + BM - 1) / BM;
    const int blocks = n_qt * d.Hq * d.B;
    const int total = (blocks + 7) & ~7;
    attend_bf16_kernel<NW><<<dim3(total), dim3(64 * NW), 0, s>>>(
        d, scale * 1.44269504088896340736f, n_qt, total, (const uint16_t*)Q, (const uint16_t*)K,
        (const uint16_t*)V, kept_idx, (uint16_t*)O);
    return hipGetLastError();
}

}  // namespace tf
