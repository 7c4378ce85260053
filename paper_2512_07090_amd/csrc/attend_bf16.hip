// Causal softmax attention over the kept tokens, bf16 inputs (Section 3.2: the tokens that
// are not skipped attend as usual and a skipped token's attention output is zero; here both
// queries and keys are the kept tokens, addressed through kept_idx, so "causal" means key rank
// <= query rank in the compacted order).
//
// Flash-style kernel for gfx950.  One work item covers 256 kept queries: 8 / U waves, each
// owning U sub-tiles of 32 queries (U = 1: two waves per SIMD, 256 registers each; U = 2: one
// wave per SIMD with the whole register file and half the LDS traffic).  It walks the key tiles
// (64 kept keys) once, K and V rows gathered through kept_idx into LDS (row-major, two stages
// each).
//   S^T = K Q^T   v_mfma_f32_32x32x16_bf16, A = K rows from LDS, B = Q fragments held in
//                 registers for the whole kernel.  The transposed product puts one query per
//                 lane column, so the online-softmax row statistics need a single cross-lane
//                 exchange (lane <-> lane + 32) per step.
//   O^T += V^T P^T  A = V^T fragments read from the row-major V tile with the LDS transpose
//                 read (ds_read_b64_tr_b16), B = P^T converted to bf16 straight from the S^T
//                 accumulator registers.  The contraction order over keys is permuted the same
//                 way for both operands (accumulator register v of a 32-key block is key
//                 8 (v / 4) + 4 (lane / 32) + v % 4), which is free because a sum is taken.
//   softmax       fp32, base 2 (scale * log2 e folded into one FMA per score), running max
//                 only moved when it grows by more than 2^8 so the O rescale is rare.
//   pipeline      The math advances in steps of 32 keys.  Scores run one step ahead of the
//                 rest and LDS fragment reads one block ahead of their MFMAs, so every MFMA
//                 block has independent VALU and LDS work next to it:
//                   block 1: S(h + 1) = K Q^T  ||  P = exp2(S(h) - max), sums, bf16
//                            ||  read V(h) fragments
//                   block 2: O += P V(h)       ||  causal mask and row max of S(h + 1)
//                            ||  read K(h + 2) fragments
//                 Tiles travel global -> registers -> LDS two iterations ahead of their use
//                 (two register sets), so an L2 miss has two iterations to arrive.
//   zero rows     The rows of the filtered positions between a query and the next kept token
//                 are written as zeros together with the query's row (kept_idx is ascending).
//   scheduling    One persistent workgroup per CU walks a static list of pairs of query tiles
//                 (tile p with tile n_qt - 1 - p: equal causal work); see the kernel.
#include "tf_kernels.h"
#include <algorithm>

// build-time choice of the work decomposition (see the kernel)
#ifndef TF_ATTEND_NW
#define TF_ATTEND_NW 8
#endif
#ifndef TF_ATTEND_DEPTH
#define TF_ATTEND_DEPTH 2
#endif

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
constexpr int kOStr = kHeadDim + 8;      // output staging row stride, elements
constexpr float kMaxSlack = 8.0f;        // running max may lag the true max by 2^8
constexpr float kMasked = -1e30f;

// LDS transpose read: inside each group of 16 lanes, lane i receives element i % 4 of the
// four 8-byte rows addressed by lanes i / 4, i / 4 + 4, i / 4 + 8, i / 4 + 12.
__device__ __forceinline__ i16x4 lds_read_tr16(const uint16_t* p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (__attribute__((address_space(3))) i16x4*)(p));
}

// The 16-byte chunks a thread moves per tile of one tensor, and the kept positions of their
// rows.  Plain members (no arrays) and by-value passing keep them in registers.
template <int CH>
struct Rows;
template <>
struct Rows<2> { uint4 r0, r1; };
template <>
struct Rows<4> { uint4 r0, r1, r2, r3; };
template <int CH>
struct Pos;
template <>
struct Pos<2> { int p0, p1; };
template <>
struct Pos<4> { int p0, p1, p2, p3; };

__device__ __forceinline__ Pos<2> load_pos(const int32_t* idx, int j, int step, int last, Pos<2>*)
{
    return Pos<2>{idx[min(j, last)], idx[min(j + step, last)]};
}
__device__ __forceinline__ Pos<4> load_pos(const int32_t* idx, int j, int step, int last, Pos<4>*)
{
    return Pos<4>{idx[min(j, last)], idx[min(j + step, last)], idx[min(j + 2 * step, last)],
                  idx[min(j + 3 * step, last)]};
}
// One 16-byte chunk of the row at position `pos`: `base` is uniform over the workgroup (the
// (batch, head) slice plus nothing else), the lane's part is a 32-bit byte offset
// pos * row_bytes + col_bytes formed by one 24-bit multiply-add (the launcher checks that a
// slice spans less than 4 GiB and that positions and row strides stay below 2^24).
__device__ __forceinline__ uint4 load16(const char* base, int pos, unsigned row_bytes, unsigned col_bytes)
{
    const unsigned off = __umul24((unsigned)pos, row_bytes) + col_bytes;
    return *reinterpret_cast<const uint4*>(base + off);
}
__device__ __forceinline__ Rows<2> load_rows(const char* base, Pos<2> p, unsigned rb, unsigned cb)
{
    return Rows<2>{load16(base, p.p0, rb, cb), load16(base, p.p1, rb, cb)};
}
__device__ __forceinline__ Rows<4> load_rows(const char* base, Pos<4> p, unsigned rb, unsigned cb)
{
    return Rows<4>{load16(base, p.p0, rb, cb), load16(base, p.p1, rb, cb), load16(base, p.p2, rb, cb),
                   load16(base, p.p3, rb, cb)};
}
// Two floats rounded to bf16 and packed into one register (v_cvt_pk_bf16_f32), and the sum of
// such a pair added to `acc` (v_dot2_f32_bf16 against (1, 1)).  The words are handled as plain
// unsigned values and only the assembled operand is reinterpreted as eight bf16 values:
// extracting words from a bf16 vector after element-wise stores made this compiler read the
// first word four times.
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ unsigned pack_bf16x2(float a, float b)
{
    const f32x2 v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float add_bf16x2(unsigned w, float acc)
{
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w),
                                           __builtin_bit_cast(bf16x2, 0x3f803f80u), acc, false);
}

// 16 bytes to global memory with the non-temporal hint (the line is not kept in the L2)
__device__ __forceinline__ void store_streaming(uint16_t* dst, uint4 v)
{
    __builtin_nontemporal_store(__builtin_bit_cast(u32x4, v), reinterpret_cast<u32x4*>(dst));
}

__device__ __forceinline__ void store_rows(Rows<2> r, uint16_t* dst, int step)
{
    *reinterpret_cast<uint4*>(dst) = r.r0;
    *reinterpret_cast<uint4*>(dst + step) = r.r1;
}
__device__ __forceinline__ void store_rows(Rows<4> r, uint16_t* dst, int step)
{
    *reinterpret_cast<uint4*>(dst) = r.r0;
    *reinterpret_cast<uint4*>(dst + step) = r.r1;
    *reinterpret_cast<uint4*>(dst + 2 * step) = r.r2;
    *reinterpret_cast<uint4*>(dst + 3 * step) = r.r3;
}

// NW: waves per workgroup, each owning 32 queries of a work item of 32 NW queries.  NW = 8: one
// workgroup per CU; NW = 4: two independent workgroups per CU (two waves per SIMD either way,
// 256 registers each), so that one workgroup's start-up, epilogue and diagonal tiles overlap
// with the other's tile loop.  DEPTH: register sets a tile passes through on its way from
// global memory to LDS, i.e. how many iterations ahead of its LDS write a tile is requested.
template <int NW, int DEPTH>
__global__ __launch_bounds__(64 * NW, 2) void attend_bf16_kernel(
    Dims d, float scale_log2, int n_qt, int n_xcd, const uint16_t* __restrict__ Q,
    const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    const int32_t* __restrict__ kept_idx, uint16_t* __restrict__ O,
    const int32_t* __restrict__ counts, long long idx_stride)
{
    constexpr int U = 1;           // 32-query sub-tiles per wave
    constexpr int NT = 64 * NW;    // threads
    constexpr int CH = 1024 / NT;  // 16-byte chunks per thread per tensor per tile
    constexpr int WQ = 32 * U;     // queries per wave
    constexpr int kBM = WQ * NW;   // kept queries per work item
    __shared__ __attribute__((aligned(16))) uint16_t smem[2 * kKTile + 2 * kVTile];
    uint16_t* const k_lds = smem;               // 2 stages of K
    uint16_t* const v_lds = smem + 2 * kKTile;  // 2 stages of V
    // Output staging of its own (145 KB of LDS in all): a wave stages and writes its rows without
    // a workgroup barrier on either side, so the waves leave an item, and start on the next
    // item's first loads, as each gets there.
    __shared__ __attribute__((aligned(16))) uint16_t ostage[kBM * kOStr];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform: branches on it are scalar

    // Persistent workgroups, one per CU, with a static schedule.  (Left to the hardware
    // dispatcher, one workgroup per query tile, CUs sit idle for many microseconds whenever a
    // workgroup ends: it hands out workgroups in order, and the durations of causal query tiles
    // differ by a factor of n_qt.)  The (batch, head) groups are split into n_xcd contiguous
    // runs, one per XCD (the count is the device's, read by the host), so an XCD's L2 holds the
    // K and V of the few groups it is working on.  Correctness does not depend on where a
    // workgroup really runs, only the L2 hit rate does.
    const int n_groups = d.B * d.Hq;
    // Static schedule: workgroup j of XCD x (x = id % n_xcd, as the dispatcher deals them) walks
    // entries j, j + W, ... of the XCD's list of (group, pair of query tiles); a pair joins
    // query tile p with n_qt - 1 - p, so every entry is the same amount of causal work, and the
    // workgroups that share a group start on it together and stream the same K / V tiles.
    const int x = blockIdx.x % n_xcd, j = blockIdx.x / n_xcd;
    const int nwx = (gridDim.x + n_xcd - 1 - x) / n_xcd;  // workgroups whose id % n_xcd is x
    const int g_lo = x * n_groups / n_xcd;
    const int ng = (x + 1) * n_groups / n_xcd - g_lo;
    const int n_pairs = (n_qt + 1) >> 1;
    const int n_entries = ng * n_pairs;

    // Ragged rows (counts != null: every batch row has its own number of kept tokens, read here
    // on the device; n_qt is only the bound for the longest possible row): the XCD's list holds,
    // group after group, as many pairs as the group's row needs (one entry for an empty row,
    // which only has zero rows to write), so that, as in the uniform case, workgroups with
    // neighbouring ids work on the same group.  (rb, row_e0): the batch row the current entry
    // lies in and the first entry of that row; entries only move forward.
    //
    // Uniform rows, last round: when the entries do not fill a whole number of rounds and the
    // rest (L entries) is at most half a round, those L entries are not dealt as pairs, which
    // would keep every other workgroup idle for a whole pair: they are the MIDDLE pairs of the
    // last L groups (the pair whose two tiles are closest in work), taken out of the list of
    // whole rounds, and their 2 L tiles go to workgroups 0 .. 2 L - 1, one tile each (two
    // neighbours share a group).  The last round then lasts one middle tile instead of a pair.
    const int full_rounds = n_entries / nwx;
    const int rest = n_entries - full_rounds * nwx;
    const bool split_rest = !counts && rest > 0 && 2 * rest <= nwx && rest <= ng && n_pairs >= 2 && (n_qt & 1) == 0;
    const int n_main = split_rest ? n_entries - rest : n_entries;  // entries dealt as pairs
    const int whole_groups = split_rest ? ng - rest : ng;          // groups that keep all their pairs
    int rb = g_lo / d.Hq, row_e0 = 0;
    for (int it = 0;; ++it) {
    const int e = j + (it >> 1) * nwx;
    int pr, bh, m, nq;
    bool single = false;  // this entry is one tile of a split middle pair
    if (counts) {
        int P = 1;
        bool done = false;
        for (;;) {
            const int lo = max(g_lo, rb * d.Hq), hi = min(g_lo + ng, (rb + 1) * d.Hq);
            if (rb >= d.B || hi <= lo) { done = true; break; }
            m = __builtin_amdgcn_readfirstlane(counts[rb]);  // kept tokens of this row
            nq = (m + kBM - 1) / kBM;                        // its query tiles
            P = m == 0 ? 1 : (nq + 1) >> 1;
            if (e < row_e0 + (hi - lo) * P) break;
            row_e0 += (hi - lo) * P;
            ++rb;
        }
        if (done) break;
        const int el = e - row_e0;
        bh = max(g_lo, rb * d.Hq) + el / P;
        pr = el % P;
    } else {
        m = d.m;
        nq = n_qt;
        if (e < n_main) {
            const int e_whole = whole_groups * n_pairs;  // entries of the groups with all pairs
            if (e < e_whole) {
                pr = e % n_pairs;
                bh = g_lo + e / n_pairs;
            } else {  // the last groups have given their middle pair away
                pr = (e - e_whole) % (n_pairs - 1);
                bh = g_lo + whole_groups + (e - e_whole) / (n_pairs - 1);
            }
        } else {
            // past the whole rounds: one tile of a middle pair, or nothing
            if (!split_rest || (it >> 1) != full_rounds || (it & 1) || j >= 2 * rest) break;
            single = true;
            pr = n_pairs - 1;
            bh = g_lo + whole_groups + (j >> 1);
        }
    }
    const int b = bh / d.Hq, hq = bh % d.Hq;
    const int hk = hq / (d.Hq / d.Hkv);
    if (m == 0) {
        // a row without kept tokens: nothing attends, every output row is zero
        if (pr == 0 && !(it & 1)) {
            uint16_t* Oz = O + (long long)b * d.os[0] + (long long)hq * d.os[1] + 8 * (tid & 15);
            for (int g = tid >> 4; g < d.n; g += NT / 16)
                *reinterpret_cast<uint4*>(Oz + (long long)g * d.os[2]) = make_uint4(0, 0, 0, 0);
        }
        continue;
    }
    if (pr >= (nq + 1) >> 1) continue;
    const int qt = single ? ((j & 1) ? pr : nq - 1 - pr) : ((it & 1) ? pr : nq - 1 - pr);
    if (!single && (it & 1) && pr == nq - 1 - pr) continue;  // the middle tile of an odd count is alone

    const int32_t* idx = kept_idx + (long long)b * idx_stride;
    const uint16_t* Qb = Q + (long long)b * d.qs[0] + (long long)hq * d.qs[1];
    const char* Kb = reinterpret_cast<const char*>(K + (long long)b * d.kvs[0] + (long long)hk * d.kvs[1]);
    const char* Vb = reinterpret_cast<const char*>(V + (long long)b * d.kvs[0] + (long long)hk * d.kvs[1]);
    uint16_t* Ob = O + (long long)b * d.os[0] + (long long)hq * d.os[1];
    const unsigned kv_row_bytes = (unsigned)d.kvs[2] * 2u;

    const int col = lane & 31, hh = lane >> 5;

    const int i0 = qt * kBM;
    // Waves w and w + NT / 256 share a SIMD.  Causal work grows with the row block, so the
    // second half of the waves takes the row blocks in reverse: every SIMD then carries one
    // early and one late block and the four SIMDs finish together.
    constexpr int NWV = NT / 64;
    const int blk = wave < NWV / 2 ? wave : NWV + NWV / 2 - 1 - wave;
    const int iw = i0 + WQ * blk;    // first query rank of this wave
    const int i_last = min(i0 + kBM, m) - 1;
    const int n_kt = i_last / kBN + 1;
    const int m_last = m - 1;
    // last key rank each of this lane's queries (one per sub-tile) may see
    int lim[U];
#pragma unroll
    for (int u = 0; u < U; ++u) lim[u] = min(iw + 32 * u + col, m_last);

    // tile-load roles: chunk i of a thread covers row tid / 16 + (NT / 16) i, columns
    // 8 (tid % 16) ..+7.  Rows past the last kept token re-read the last kept row: finite
    // values that the mask turns into zero weights, so the loads need no branch.
    const int row0 = tid >> 4;
    const int col0 = (tid & 15) * 8;
    constexpr int RS = NT / 16;  // row step between a thread's chunks
    Rows<CH> kreg_a, vreg_a, kreg_b, vreg_b;
    Pos<CH> pos_k, pos_v, pos_n;
#define TF_LOAD_IDX(P, J0) P = load_pos(idx, (J0) + row0, RS, m_last, (Pos<CH>*)nullptr)
#define TF_LOAD_ROWS(R, BASE, P) R = load_rows(BASE, P, kv_row_bytes, 2u * col0)
#define TF_STORE_ROWS(R, STAGE, STRIDE) store_rows(R, (STAGE) + row0 * (STRIDE) + col0, RS * (STRIDE))
#define TF_COPY_POS(DST, SRC) DST = SRC

    // ---- prologue, part 1: every index first, then every row load, no wait in between -----
    int qpos[U];   // positions of this lane's queries
#pragma unroll
    for (int u = 0; u < U; ++u) qpos[u] = idx[lim[u]];
    Pos<CH> pos_0, pos_1;
    {
        // (opaque copy of the row number: these index sets do not depend on the item, and
        // would otherwise be kept in registers, or spilled, across the whole item loop)
        int row0p = row0;
        asm volatile("" : "+v"(row0p));
        pos_0 = load_pos(idx, row0p, RS, m_last, (Pos<CH>*)nullptr);
        pos_1 = load_pos(idx, kBN + row0p, RS, m_last, (Pos<CH>*)nullptr);
        // rows of the tiles iteration 0 requests: V(DEPTH) and K(DEPTH + 1)
        pos_v = load_pos(idx, DEPTH * kBN + row0p, RS, m_last, (Pos<CH>*)nullptr);
        pos_k = load_pos(idx, (DEPTH + 1) * kBN + row0p, RS, m_last, (Pos<CH>*)nullptr);
    }
    // Q fragments (B operand of S^T = K Q^T): for sub-tile u, lane (col, hh) holds, for
    // k-step s, the 8 elements 16 s + 8 hh .. +7 of query row iw + 32 u + col.
    bf16x8 qf[U][8];
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const uint16_t* src = Qb + (long long)qpos[u] * d.qs[2];
#pragma unroll
        for (int s = 0; s < 8; ++s)
            qf[u][s] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4*>(src + 16 * s + 8 * hh));
    }
    TF_LOAD_ROWS(kreg_a, Kb, pos_0);  // K(0)
    TF_LOAD_ROWS(vreg_a, Vb, pos_0);  // V(0)
    TF_LOAD_ROWS(kreg_b, Kb, pos_1);  // K(1)
    if constexpr (DEPTH == 2) TF_LOAD_ROWS(vreg_b, Vb, pos_1);  // V(1), stays in registers until iteration 0 ends
    TF_STORE_ROWS(kreg_a, k_lds, kKStr);
    TF_STORE_ROWS(vreg_a, v_lds, kVStr);
    TF_STORE_ROWS(kreg_b, k_lds + kKTile, kKStr);
    if constexpr (DEPTH == 2) TF_LOAD_ROWS(kreg_a, Kb, pos_v);  // K(2), stays in flight
    __syncthreads();

    // LDS offsets of this lane's operand fragments inside a K / V stage
    const int k_off = col * kKStr + 8 * hh;
    const int v_off = (4 * hh + ((lane & 15) >> 2)) * kVStr + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    f32x16 oacc[U][4];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[u][dt][v] = 0.f;
    float m_run[U];  // running max of the RAW scores (may lag, see kMaxSlack)
    float l_run[U];  // this lane's share of the softmax denominators, in two independent
    float l_alt[U];  // chains (even / odd pairs of keys)
#pragma unroll
    for (int u = 0; u < U; ++u) {
        m_run[u] = kMasked;
        l_run[u] = 0.f;
        l_alt[u] = 0.f;
    }

    bf16x8 kf[8];           // K fragments of the 32 keys whose scores are computed next
    bf16x8 vf[2][4];        // V^T fragments of the 32 keys being accumulated
    bf16x8 pf[U][2];        // P^T of the current step, per sub-tile and 16-key k-step
    f32x16 s_x[U], s_y[U];  // raw scores of two consecutive steps, per sub-tile

    // K fragments of the 32 keys whose first row sits at `ks` in a K stage
    auto read_kf = [&](const uint16_t* ks) {
#pragma unroll
        for (int s = 0; s < 8; ++s) kf[s] = *reinterpret_cast<const bf16x8*>(ks + k_off + 16 * s);
    };
    // V^T fragments of the 32 keys starting at `vs`: k-slot e of k-step ks is key
    // 16 ks + 8 (e / 4) + 4 hh + e % 4, matching the P^T operand
    auto read_vf = [&](const uint16_t* vs) {
#pragma unroll
        for (int ks2 = 0; ks2 < 2; ++ks2)
#pragma unroll
            for (int dt = 0; dt < 4; ++dt) {
                const uint16_t* vp = vs + v_off + 16 * ks2 * kVStr + 32 * dt;
                const i16x4 both[2] = {lds_read_tr16(vp), lds_read_tr16(vp + 8 * kVStr)};
                vf[ks2][dt] = __builtin_bit_cast(bf16x8, both);
            }
    };
    // raw scores of 32 keys from the fragments in kf
    const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#define TF_QK(S)                                                                               \
    _Pragma("unroll") for (int u = 0; u < U; ++u)                                              \
        S[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[0], qf[u][0], zero16, 0, 0, 0);      \
    _Pragma("unroll") for (int s = 1; s < 8; ++s)                                              \
        _Pragma("unroll") for (int u = 0; u < U; ++u)                                          \
            S[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[s], qf[u][s], S[u], 0, 0, 0)
    // causal / tail mask of the 32 keys starting at rank j0, then the row max.
    // Accumulator register v is key j0 + 8 (v / 4) + 4 hh + v % 4.
    auto mask_and_max = [&](f32x16& sacc, int j0, int limit, bool need_mask) -> float {
        if (need_mask) {
            const int t = j0 + 4 * hh - limit;  // key rank of register 0 minus the limit
#pragma unroll
            for (int v = 0; v < 16; ++v)
                if (t + (8 * (v >> 2) + (v & 3)) > 0) sacc[v] = kMasked;
        }
        // two chains of three-operand maxima
        float mx = fmaxf(sacc[0], sacc[1]), my = fmaxf(sacc[2], sacc[3]);
#pragma unroll
        for (int v = 4; v < 16; v += 4) {
            mx = fmaxf(fmaxf(mx, sacc[v]), sacc[v + 1]);
            my = fmaxf(fmaxf(my, sacc[v + 2]), sacc[v + 3]);
        }
        mx = fmaxf(mx, my);
        // the other half of this query's keys sits 32 lanes away: swap halves in the VALU
        const FloatPair sw = swap32(mx, mx);
        return fmaxf(sw.first, sw.second);
    };
    // Move a running max when the new max exceeds it by more than the slack; rescale what
    // has been accumulated so far for that sub-tile.
    auto update_max = [&](int u, float mx) {
        const bool grow = (mx - m_run[u]) * scale_log2 > kMaxSlack;
        if (__any(grow)) {
            const float m_new = grow ? mx : m_run[u];
            const float corr = __builtin_amdgcn_exp2f((m_run[u] - m_new) * scale_log2);
            m_run[u] = m_new;
            l_run[u] *= corr;
            l_alt[u] *= corr;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int v = 0; v < 16; ++v) oacc[u][dt][v] *= corr;
        }
    };

    // One step over 32 keys.  On entry S_CUR holds the masked raw scores of step h and kf the
    // K fragments of step h + 1; VS is where V(h) sits in LDS, KS_NEXT where K(h + 2) sits;
    // J_NEXT is the key rank at which step h + 1 starts.  (A macro: the score registers must
    // not be reached through pointer arguments.)
#define TF_STEP(S_CUR, S_NXT, VS, KS_NEXT, J_NEXT, MASK_NEXT)                                   \
    do {                                                                                       \
        /* block 1 */                                                                          \
        read_vf(VS);                                                                           \
        TF_QK(S_NXT);                                                                          \
        _Pragma("unroll") for (int u = 0; u < U; ++u) {                                        \
            const float mc = m_run[u] * scale_log2;                                            \
            float p_[16];                                                                      \
            _Pragma("unroll") for (int v = 0; v < 16; ++v)                                     \
                p_[v] = __builtin_amdgcn_exp2f(fmaf(S_CUR[u][v], scale_log2, -mc));            \
            /* the denominator sums the weights AS ROUNDED for the matrix product, so every */ \
            /* output row is an exact convex combination of value rows                      */ \
            _Pragma("unroll") for (int ks2 = 0; ks2 < 2; ++ks2) {                              \
                u32x4 w_;                                                                      \
                _Pragma("unroll") for (int i = 0; i < 4; ++i) {                                \
                    w_[i] = pack_bf16x2(p_[8 * ks2 + 2 * i], p_[8 * ks2 + 2 * i + 1]);         \
                    if (i & 1) l_alt[u] = add_bf16x2(w_[i], l_alt[u]);                         \
                    else l_run[u] = add_bf16x2(w_[i], l_run[u]);                               \
                }                                                                              \
                pf[u][ks2] = __builtin_bit_cast(bf16x8, w_);                                   \
            }                                                                                  \
        }                                                                                      \
        /* block 2 */                                                                          \
        read_kf(KS_NEXT);                                                                      \
        _Pragma("unroll") for (int ks2 = 0; ks2 < 2; ++ks2)                                    \
            _Pragma("unroll") for (int dt = 0; dt < 4; ++dt)                                   \
                _Pragma("unroll") for (int u = 0; u < U; ++u)                                  \
                    oacc[u][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                     \
                        vf[ks2][dt], pf[u][ks2], oacc[u][dt], 0, 0, 0);                        \
        float mx_[U];                                                                          \
        _Pragma("unroll") for (int u = 0; u < U; ++u)                                          \
            mx_[u] = mask_and_max(S_NXT[u], J_NEXT, lim[u], MASK_NEXT);                        \
        _Pragma("unroll") for (int u = 0; u < U; ++u) update_max(u, mx_[u]);                   \
    } while (0)

    // ---- prologue, part 2: scores of step 0; K fragments of step 1 ------------------------
    {
        const bool diag0 = kBN > iw || kBN > m;
        read_kf(k_lds);
        TF_QK(s_x);
#pragma unroll
        for (int u = 0; u < U; ++u) update_max(u, mask_and_max(s_x[u], 0, lim[u], diag0));
        read_kf(k_lds + 32 * kKStr);
    }
    __syncthreads();  // K(0) is fully in registers before iteration 0 may overwrite its stage

    // Iteration kt: issue the loads of K(kt + 1 + DEPTH) and V(kt + DEPTH) into register set LD,
    // do the two steps of tile kt, then write set ST (K(kt + 2), V(kt + 1); with DEPTH = 2 issued
    // one iteration earlier into the other set, with DEPTH = 1 the loads just issued) into the
    // stages that K(kt) and V(kt - 1) have left.  Index loads go first so that waiting for them
    // leaves the row loads in flight.
#define TF_ITERATION(KT, LD_K, LD_V, ST_K, ST_V)                                                \
    do {                                                                                       \
        const int cur = (KT) & 1;                                                              \
        const int j0 = (KT) * kBN;                                                             \
        TF_LOAD_IDX(pos_n, j0 + (2 + DEPTH) * kBN);                                            \
        TF_LOAD_ROWS(LD_K, Kb, pos_k);                                                         \
        TF_LOAD_ROWS(LD_V, Vb, pos_v);                                                         \
        TF_COPY_POS(pos_v, pos_k);                                                             \
        TF_COPY_POS(pos_k, pos_n);                                                             \
        if (j0 <= iw) {                                                                        \
            const uint16_t* vs = v_lds + cur * kVTile;                                         \
            const uint16_t* kn = k_lds + (cur ^ 1) * kKTile;         /* K(kt + 1) */           \
            const bool m1 = j0 + kBN > iw || j0 + kBN > m;           /* this tile is masked */ \
            const bool m2 = j0 + 2 * kBN > iw || j0 + 2 * kBN > m;   /* the next one is */     \
            TF_STEP(s_x, s_y, vs, kn, j0 + 32, m1);                                            \
            TF_STEP(s_y, s_x, vs + 32 * kVStr, kn + 32 * kKStr, j0 + kBN, m2);                 \
        }                                                                                      \
        TF_STORE_ROWS(ST_K, k_lds + cur * kKTile, kKStr);                                      \
        TF_STORE_ROWS(ST_V, v_lds + (cur ^ 1) * kVTile, kVStr);                                \
        __syncthreads();                                                                       \
    } while (0)

    // after the prologue, DEPTH = 2: kreg_a = K(2) is in flight, vreg_b = V(1) is loaded
    for (int kt = 0; kt < n_kt; kt += 2) {
        if constexpr (DEPTH == 2) {
            TF_ITERATION(kt, kreg_b, vreg_a, kreg_a, vreg_b);
            if (kt + 1 < n_kt) TF_ITERATION(kt + 1, kreg_a, vreg_b, kreg_b, vreg_a);
        } else {
            TF_ITERATION(kt, kreg_a, vreg_a, kreg_a, vreg_a);
            if (kt + 1 < n_kt) TF_ITERATION(kt + 1, kreg_a, vreg_a, kreg_a, vreg_a);
        }
    }
#undef TF_ITERATION
#undef TF_STEP
#undef TF_QK
#undef TF_LOAD_IDX
#undef TF_LOAD_ROWS
#undef TF_STORE_ROWS
#undef TF_COPY_POS

    // normalise, transpose through LDS and write whole rows
    // (the lane number goes through an opaque move so that the addresses below are formed
    // here, per item, instead of being carried in registers across the tile loop)
    int ln = lane;
    asm volatile("" : "+v"(ln));
    uint16_t* os = ostage + wave * (WQ * kOStr);  // [WQ queries][kOStr], this wave's alone
#pragma unroll
    for (int u = 0; u < U; ++u) {
        const float l_mine = l_run[u] + l_alt[u];
        const float l_tot = l_mine + __shfl_xor(l_mine, 32);
        const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
#pragma unroll
        for (int dt = 0; dt < 4; ++dt)
#pragma unroll
            for (int v4 = 0; v4 < 4; ++v4) {
                bf16x4 o4;
#pragma unroll
                for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(oacc[u][dt][4 * v4 + e] * inv);
                *reinterpret_cast<bf16x4*>(os + (32 * u + (ln & 31)) * kOStr + 32 * dt + 8 * v4 + 4 * (ln >> 5)) = o4;
            }
    }
    // the rows are read back by other lanes of this wave only: LDS operations of one wave
    // complete in order, the compiler must just not move them across this point
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    // Every 16-lane group writes one query's row: four rows per store instruction.
    const uint4 zero4 = make_uint4(0, 0, 0, 0);
    uint16_t* const Oc = Ob + 8 * (ln & 15);  // this lane's 16-byte column
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
        for (int it = 0; it < 8; ++it) {
            const int r = 4 * it + (ln >> 4);  // query row inside the sub-tile
            const int p = __shfl(qpos[u], r);    // its position, held by lane r
            if (iw + 32 * u + r < m) {
                const uint4 v = *reinterpret_cast<const uint4*>(os + (32 * u + r) * kOStr + 8 * (ln & 15));
                store_streaming(Oc + (long long)p * d.os[2], v);
            }
        }
    // The zero rows this wave owns: the filtered positions after its first query and before the
    // first query of the next wave (n after the last kept token).  They are written densely, four
    // rows per store instruction whatever the gaps look like: with z_i = the zero rows before
    // query i (= position_i - position_0 - i, ascending), the k-th zero row sits at
    // position_0 + 1 + k + #{i >= 1 : z_i <= k}, and the count is a ballot over the queries.
    // All output stores are non-temporal: O is written once and never read here, and lines of O
    // allocated in the L2 push out K / V tiles that other query tiles of the group still need.
    static_assert(U == 1, "the dense zero-row writer assumes one 32-query sub-tile per wave");
    {
        const int n_valid = min(max(m - iw, 0), WQ);  // queries of this wave that exist
        if (n_valid > 0) {
            const int p_first = __builtin_amdgcn_readfirstlane(qpos[0]);
            const int last_rank = iw + n_valid - 1;
            const int p_end = last_rank < m_last ? idx[last_rank + 1] : d.n;  // uniform
            const int n_zero = __builtin_amdgcn_readfirstlane(p_end - p_first - n_valid);
            const int z_mine = qpos[0] - p_first - ln;  // meaningful for lanes 1 .. n_valid - 1
            const bool counted = ln >= 1 && ln < n_valid;
            const int grp = ln >> 4;
            for (int k0 = 0; k0 < n_zero; k0 += 4) {
                const int c0 = __popcll(__ballot(counted && z_mine <= k0));
                const int c1 = __popcll(__ballot(counted && z_mine <= k0 + 1));
                const int c2 = __popcll(__ballot(counted && z_mine <= k0 + 2));
                const int c3 = __popcll(__ballot(counted && z_mine <= k0 + 3));
                const int cnt = grp == 0 ? c0 : (grp == 1 ? c1 : (grp == 2 ? c2 : c3));
                const int k = k0 + grp;
                if (k < n_zero)
                    store_streaming(Oc + (long long)(p_first + 1 + k + cnt) * d.os[2], zero4);
            }
        }
    }
    // positions before the first kept token
    if (qt == 0 && blk == 0) {
        const int ze = __shfl(qpos[0], 0);
        for (int g = ln >> 4; g < ze; g += 4) *reinterpret_cast<uint4*>(Oc + (long long)g * d.os[2]) = zero4;
    }
    // (no barrier here: the last tile-loop iteration ended with one, after which nobody reads a
    // tile stage, and the staging area is not shared)
    }  // items
}

}  // namespace

hipError_t launch_attend_bf16(const Dims& d, float scale, const void* Q, const void* K,
                              const void* V, const int32_t* kept_idx, void* O, int n_cu, int n_xcd,
                              const int32_t* counts, long long idx_stride, hipStream_t s)
{
    // the tile gathers address a row as a 32-bit byte offset from its (batch, head) slice
    if (d.n > (1 << 24) || d.kvs[2] * 2 >= (1 << 24) || (long long)d.n * d.kvs[2] * 2 >= (1ll << 32))
        return hipErrorInvalidValue;
    n_xcd = std::max(n_xcd, 1);
    // with per-row counts d.m is the bound (the longest possible row)
    constexpr int NW = TF_ATTEND_NW, DEPTH = TF_ATTEND_DEPTH;
    constexpr int kBM = 32 * NW, wg_per_cu = 8 / NW;
    const int n_qt = (d.m + kBM - 1) / kBM;
    const long long items = (long long)d.B * d.Hq * n_qt;
    // persistent workgroups: as many as are resident at once; at least one per XCD, so that every
    // residue of id % n_xcd owns a share of the groups
    const int grid = (int)std::max<long long>(n_xcd, std::min<long long>(items, (long long)wg_per_cu * std::max(n_cu, 1)));
    attend_bf16_kernel<NW, DEPTH><<<dim3(grid), dim3(64 * NW), 0, s>>>(
        d, scale * 1.44269504088896340736f, n_qt, n_xcd, (const uint16_t*)Q,
        (const uint16_t*)K, (const uint16_t*)V, kept_idx, (uint16_t*)O, counts,
        counts ? idx_stride : (long long)d.m);
    return hipGetLastError();
}

}  // namespace tf
