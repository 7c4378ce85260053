// Causal softmax attention over the kept tokens, bf16 inputs (Section 3.2: the tokens that
// are not skipped attend as usual; here both queries and keys are the kept tokens, addressed
// through kept_idx, so "causal" means key rank <= query rank in the compacted order).
//
// Flash-style kernel for gfx950.  One workgroup = NW waves x 32 kept queries; it walks the key
// tiles (64 kept keys) once, K and V rows gathered through kept_idx into LDS (row-major,
// two stages each).
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
//   pipeline      The math advances in halves of a tile (32 keys), the scores running one half
//                 ahead of the rest, so that every MFMA block has independent VALU work next
//                 to it and the matrix and vector pipes overlap inside one wave:
//                   S(next half) = K Q^T  ||  P = exp2(S(this half) - max), row sums, bf16
//                   O += P V(this half)   ||  causal mask and row max of S(next half)
//                 K sits in three LDS stages (K(kt) second half and K(kt+1) first half are read
//                 while K(kt+2) lands), V in two; the next tiles travel from global memory to
//                 registers during the iteration and are written to LDS at its end.
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
constexpr float kMaxSlack = 8.0f;        // running max may lag the true max by 2^8
constexpr float kMasked = -1e30f;

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
    constexpr int CH = 1024 / NT;  // 16-byte chunks per thread per tensor per tile
    __shared__ __attribute__((aligned(16))) uint16_t smem[3 * kKTile + 2 * kVTile];
    uint16_t* const k_lds = smem;               // 3 stages of K
    uint16_t* const v_lds = smem + 3 * kKTile;  // 2 stages of V

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
    const int lim = min(iq, d.m - 1);  // last key rank this lane's query may see

    // tile-load roles: chunk c = tid + NT * i covers row c / 16, columns 8 (c % 16) ..+7.
    // Rows past the last kept token re-read the last kept row: finite values that the mask
    // turns into zero weights, so the loads need no branch.
    // Everything below is spelled out for the two chunks a thread owns (plain scalars keep the
    // in-flight tiles in registers).
    static_assert(CH == 2, "tile loads are written for 512 threads");
    const int row0 = tid >> 4, row1 = (tid + NT) >> 4;
    const int col0 = (tid & 15) * 8;  // same column slice for both chunks
    struct Rows { uint4 a, b; };      // chunk 0 / chunk 1 of one tile of one tensor
    struct Pos { int a, b; };         // kept positions of the two rows
    auto load_idx = [&](int j0) -> Pos {
        return Pos{idx[min(j0 + row0, d.m - 1)], idx[min(j0 + row1, d.m - 1)]};
    };
    auto load_rows = [&](const uint16_t* base, Pos p) -> Rows {
        return Rows{*reinterpret_cast<const uint4*>(base + (long long)p.a * s_t + col0),
                    *reinterpret_cast<const uint4*>(base + (long long)p.b * s_t + col0)};
    };
    auto store_rows = [&](Rows r, uint16_t* stage, int stride) {
        *reinterpret_cast<uint4*>(stage + row0 * stride + col0) = r.a;
        *reinterpret_cast<uint4*>(stage + row1 * stride + col0) = r.b;
    };

    // Q fragments (B operand of S^T = K Q^T): lane (col, hh) holds, for k-step s, the 8
    // elements 16 s + 8 hh .. +7 of query row `col`.
    bf16x8 qf[8];
    {
        const uint16_t* src = Qb + (long long)idx[min(iq, d.m - 1)] * d.qs[2];
#pragma unroll
        for (int s = 0; s < 8; ++s)
            qf[s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(src + 16 * s + 8 * hh));
    }

    // LDS offsets of this lane's operand fragments inside a K / V stage
    const int k_off = col * kKStr + 8 * hh;
    const int v_off = (4 * hh + ((lane & 15) >> 2)) * kVStr + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    f32x16 oacc[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int v = 0; v < 16; ++v) oacc[dt][v] = 0.f;
    float m_run = kMasked;  // running max of the RAW scores (may lag, see kMaxSlack)
    float l_run = 0.f;      // this lane's share of the softmax denominator

    // raw scores S^T (32 keys x 32 queries) of half a tile; ks points at the half's first row
    auto qk_half = [&](f32x16& sacc, const uint16_t* ks) {
#pragma unroll
        for (int v = 0; v < 16; ++v) sacc[v] = 0.f;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(ks + k_off + 16 * s);
            sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], sacc, 0, 0, 0);
        }
    };
    // causal / tail mask of the 32 keys starting at rank j0, then their row max.
    // Accumulator register v is key j0 + 8 (v / 4) + 4 hh + v % 4.
    auto mask_and_max = [&](f32x16& sacc, int j0) -> float {
        if (j0 + 31 > iw || j0 + 32 > d.m) {
            const int t = j0 + 4 * hh - lim;  // key rank of register 0 minus the limit
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (t + (8 * (v >> 2) + (v & 3)) > 0) sacc[v] = kMasked;
        }
        float mx = sacc[0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sacc[v]);
        return fmaxf(mx, __shfl_xor(mx, 32));
    };
    // Move the running max when the new max exceeds it by more than the slack; rescale what
    // has been accumulated so far.
    auto update_max = [&](float mx) {
        const bool grow = (mx - m_run) * scale_log2 > kMaxSlack;
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
    };
    // P = exp2((S - max) * scale), this lane's share of the row sums, P^T as bf16 B operands
    auto softmax_half = [&](const f32x16& sacc, bf16x8* pf) {
        const float mc = m_run * scale_log2;
        float psum = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float p = __builtin_amdgcn_exp2f(fmaf(sacc[v], scale_log2, -mc));
            psum += p;
            pf[v >> 3][v & 7] = (__bf16)p;
        }
        l_run += psum;
    };
    // O^T (d x queries) += V^T P^T over 32 keys; vs points at the half's first V row.
    // k-slot e of k-step ks is key 16 ks + 8 (e / 4) + 4 hh + e % 4 for both operands.
    auto pv_half = [&](const bf16x8* pf, const uint16_t* vs) {
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2) {
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const uint16_t* vp = vs + v_off + 16 * ks2 * kVStr + 32 * dt;
                const i16x4 lo = lds_read_tr16(vp);
                const i16x4 hi = lds_read_tr16(vp + 8 * kVStr);
                const i16x4 both[2] = {lo, hi};
                oacc[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, both), pf[ks2], oacc[dt], 0, 0, 0);
            }
        }
    };

    // ---- prologue: K(0), V(0), K(1) into LDS; K(2), V(1) in flight; S(0, half 0) ----------
    // Two register sets carry tiles from global memory to LDS, so a tile has two iterations
    // to arrive: iteration kt issues the loads of K(kt + 3) and V(kt + 2) into one set and, at
    // its end, writes the other set (K(kt + 2), V(kt + 1), issued one iteration earlier).
    Rows kreg_a, vreg_a, kreg_b, vreg_b;
    Pos pos_k, pos_v;  // kept positions of the rows of the next K / V tile to fetch
    pos_k = load_idx(0);
    kreg_a = load_rows(Kb, pos_k);
    vreg_a = load_rows(Vb, pos_k);
    pos_k = load_idx(kBN);
    pos_v = load_idx(2 * kBN);
    store_rows(kreg_a, k_lds, kKStr);
    store_rows(vreg_a, v_lds, kVStr);
    kreg_b = load_rows(Kb, pos_k);   // K(1)
    vreg_a = load_rows(Vb, pos_k);   // V(1), stays in flight
    kreg_a = load_rows(Kb, pos_v);   // K(2), stays in flight
    pos_k = load_idx(3 * kBN);
    store_rows(kreg_b, k_lds + kKTile, kKStr);
    __syncthreads();
    f32x16 s_x, s_y;  // scores of half 0 / half 1 of a tile
    qk_half(s_x, k_lds);
    update_max(mask_and_max(s_x, 0));

    // K stages rotate over three buffers: iteration kt reads K(kt) (its second half) and
    // K(kt + 1) (its first half) while K(kt + 2) is being written.
    int ks_cur = 0, ks_nxt = 1, ks_wr = 2;
#define TF_ISSUE_LOADS(ld_k, ld_v, kt)                                                         \
    do {                                                                                      \
        ld_k = load_rows(Kb, pos_k); /* K(kt + 3) */                                          \
        ld_v = load_rows(Vb, pos_v); /* V(kt + 2) */                                          \
        pos_v = pos_k;                                                                        \
        pos_k = load_idx(((kt) + 4) * kBN);                                                   \
    } while (0)
#define TF_FINISH(st_k, st_v, kt)                                                              \
    do {                                                                                      \
        store_rows(st_k, k_lds + ks_wr * kKTile, kKStr);            /* K(kt + 2) */           \
        store_rows(st_v, v_lds + (((kt) & 1) ^ 1) * kVTile, kVStr); /* V(kt + 1) */           \
        __syncthreads();                                                                      \
        const int t_ = ks_cur;                                                                \
        ks_cur = ks_nxt;                                                                      \
        ks_nxt = ks_wr;                                                                       \
        ks_wr = t_;                                                                           \
    } while (0)
    auto compute = [&](int kt) {
        const int j0 = kt * kBN;
        const uint16_t* vs = v_lds + (kt & 1) * kVTile;
        if (j0 + 32 <= iw) {
            bf16x8 pf[2];
            // half-step A: S(kt, 1) = K Q^T  ||  P(kt, 0); then O += P V  ||  mask, max of S(kt, 1)
            qk_half(s_y, k_lds + ks_cur * kKTile + 32 * kKStr);
            softmax_half(s_x, pf);
            pv_half(pf, vs);
            update_max(mask_and_max(s_y, j0 + 32));
            // half-step B: S(kt + 1, 0)  ||  P(kt, 1); then O += P V  ||  mask, max of S(kt + 1, 0)
            qk_half(s_x, k_lds + ks_nxt * kKTile);
            softmax_half(s_y, pf);
            pv_half(pf, vs + 32 * kVStr);
            update_max(mask_and_max(s_x, j0 + kBN));
        } else if (j0 <= iw) {
            // last tile of this wave: only its first 32 keys are visible
            bf16x8 pf[2];
            softmax_half(s_x, pf);
            pv_half(pf, vs);
        }
    };
    for (int kt = 0; kt < n_kt; kt += 2) {
        TF_ISSUE_LOADS(kreg_b, vreg_b, kt);
        compute(kt);
        TF_FINISH(kreg_a, vreg_a, kt);
        if (kt + 1 < n_kt) {
            TF_ISSUE_LOADS(kreg_a, vreg_a, kt + 1);
            compute(kt + 1);
            TF_FINISH(kreg_b, vreg_b, kt + 1);
        }
    }
#undef TF_ISSUE_LOADS
#undef TF_FINISH

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
