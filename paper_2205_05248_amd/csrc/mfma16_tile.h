// Wave-level building blocks for tiles of 16 (episode, agent) rows with 16x16x32 bf16 MFMAs.
// As with the 32-row tiles the weights are the A operand (16 output features x 32 k) and the
// activations the B operand (32 k x 16 rows).  Lane l (q = l / 16, c = l % 16):
//   A  : feature c,  k = 8 q + 0..7
//   B  : row c,      k = 8 q + 0..7
//   C  : row c,      features 4 q + 0..3      (four fp32 values)
// The accumulators of two adjacent feature blocks hold, per lane, exactly the eight values of
// one k-step of the next layer's B operand; the weight fragments of such layers are stored in
// the matching k order (pack_weights.hip), so results never leave registers between layers.
#pragma once
#include "mfma_tile.h"

namespace marl {

template <int P>
__device__ __forceinline__ void mma16(f32x4 &acc, const WFrag<P> &w, const Frag<P> &b)
{
    if constexpr (P == 2) {
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w.lo, b.hi, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w.hi, b.lo, acc, 0, 0, 0);
    }
    acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w.hi, b.hi, acc, 0, 0, 0);
}

// The same for N accumulators that share the B operand.  With two planes the three products of one accumulator
// depend on each other, and a matrix instruction issued right behind the one it depends on waits out the depth
// of the pipeline; taking each kind of product across all accumulators first keeps dependent instructions N
// apart.  Every accumulator still receives lo.hi, hi.lo, hi.hi in that order: the same bits as N calls of mma16.
template <int P, int N>
__device__ __forceinline__ void mma16_across(f32x4 *const (&acc)[N], const WFrag<P> *const (&w)[N], const Frag<P> &b)
{
    if constexpr (P == 2) {
#pragma unroll
        for (int i = 0; i < N; ++i) *acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[i]->lo, b.hi, *acc[i], 0, 0, 0);
#pragma unroll
        for (int i = 0; i < N; ++i) *acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[i]->hi, b.lo, *acc[i], 0, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < N; ++i) *acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(w[i]->hi, b.hi, *acc[i], 0, 0, 0);
}

// Feature blocks 2 j and 2 j + 1 of a result -> k-step j of the next operand.
template <int P>
__device__ __forceinline__ Frag<P> frag_of_pair(const f32x4 &even, const f32x4 &odd)
{
    const float v[8] = {even[0], even[1], even[2], even[3], odd[0], odd[1], odd[2], odd[3]};
    return to_frag<P>(v);
}

// The four per-feature table entries this lane's accumulator slots of block blk refer to.
__device__ __forceinline__ f32x4 load_feature4(const float *table, int blk, int q)
{
    return *reinterpret_cast<const f32x4 *>(table + 16 * blk + 4 * q);
}

// h' = (1 - z) n + z h on the four slots of one block.
__device__ __forceinline__ f32x4 gru_blend4(const f32x4 &ar, const f32x4 &az, const f32x4 &ain, const f32x4 &ahn, const f32x4 &h)
{
    f32x4 out;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const float rr = sigmoidf_fast(ar[r]), zz = sigmoidf_fast(az[r]);
        const float nn = tanhf_fast(ain[r] + rr * ahn[r]);
        out[r] = fmaf(zz, h[r] - nn, nn);
    }
    return out;
}

// ---- action-side helpers: a row's Q values sit in the four lanes c, c + 16, c + 32, c + 48;
// lane q holds actions 16 ab + 4 q + 0..3 of action block ab.

// One (possibly unaligned) 32-bit load per action block fetches the availability bytes of the
// lane's four actions; the address is clamped into the row (A >= 4), every load unconditional.
template <int AB>
__device__ __forceinline__ void issue_avail_loads16(const uint8_t *__restrict__ avail_row, int A, int q, uint32_t (&raw)[AB])
{
#pragma unroll
    for (int ab = 0; ab < AB; ++ab) __builtin_memcpy(&raw[ab], avail_row + min(16 * ab + 4 * q, A - 4), 4);
}

// Bit 4 ab + r is set when action 16 ab + 4 q + r exists and is available.
template <int AB>
__device__ __forceinline__ uint32_t avail_mask16(const uint32_t (&raw)[AB], int A, int q, bool valid)
{
    uint32_t mask = 0;
#pragma unroll
    for (int ab = 0; ab < AB; ++ab) {
        const int a0 = 16 * ab + 4 * q;
        const int skip = a0 - min(a0, A - 4);                  // bytes of the word that precede a0
        const uint32_t w = skip < 4 ? raw[ab] >> (8 * skip) : 0u;
#pragma unroll
        for (int i = 0; i < 4; ++i) mask |= ((w >> (8 * i)) & 0xFFu) ? (1u << (4 * ab + i)) : 0u;
    }
    return valid ? mask : 0u;
}

// Rows with fewer than four actions: all of them belong to lane quarter 0, block 0.
__device__ __forceinline__ uint32_t avail_mask_small16(const uint8_t *__restrict__ avail_row, int A, int q, bool valid)
{
    uint32_t mask = 0;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uint32_t v = avail_row[min(i, A - 1)];
        mask |= (i < A && v) ? (1u << i) : 0u;
    }
    return (valid && q == 0) ? mask : 0u;
}

// A row's Q values sit in the four lanes c, c + 16, c + 32, c + 48 (lane quarters 0..3).  The two
// swaps below hand every lane a pair of quarters' values without a trip through LDS:
// halves16: (quarter 0, quarter 1) in the lanes of quarters 0 and 1, (2, 3) in those of 2 and 3;
// halves32: (q & 1, (q & 1) + 2).  One after the other they combine all four, and every lane ends
// with the same result, the operands always in quarter order.
struct LanePair { uint32_t lower, upper; };
__device__ __forceinline__ LanePair halves16(uint32_t x)
{
    const auto r = __builtin_amdgcn_permlane16_swap(x, x, false, false);
    return {r[0], r[1]};
}
__device__ __forceinline__ LanePair halves32(uint32_t x)
{
    const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
    return {r[0], r[1]};
}
__device__ __forceinline__ uint32_t or_quarters(uint32_t x)
{
    LanePair p = halves16(x);
    p = halves32(p.lower | p.upper);
    return p.lower | p.upper;
}

// Masked argmax of a row whose Q values are split over the four lanes c, c + 16, c + 32, c + 48;
// lowest index on ties; idx = -1 when nothing is available.  The quarters are combined with lane
// swaps (vector instructions), or with LDS shuffles when VIA_LDS (see masked_max16 for when).
template <int AB, bool VIA_LDS = false>
__device__ __forceinline__ void masked_argmax16(const f32x4 (&qv)[AB], uint32_t slots, int q, float &best_q, int &best_idx)
{
    best_q = 0.0f; best_idx = -1;
#pragma unroll
    for (int ab = 0; ab < AB; ++ab)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool ok = (slots >> (4 * ab + r)) & 1u;
            if (ok && (best_idx < 0 || qv[ab][r] > best_q)) { best_q = qv[ab][r]; best_idx = 16 * ab + 4 * q + r; }
        }
    auto better = [](float qa, int ia, float qb, int ib, float &q_out, int &i_out) {      // ties: the lower index
        const bool take_b = ib >= 0 && (ia < 0 || qb > qa || (qb == qa && ib < ia));
        q_out = take_b ? qb : qa;
        i_out = take_b ? ib : ia;
    };
    if constexpr (VIA_LDS) {
#pragma unroll
        for (int d = 16; d <= 32; d *= 2) {
            const float oq = __shfl_xor(best_q, d);
            const int oi = __shfl_xor(best_idx, d);
            better(best_q, best_idx, oq, oi, best_q, best_idx);
        }
    } else {
        LanePair pq = halves16(__float_as_uint(best_q)), pi = halves16((uint32_t)best_idx);
        better(__uint_as_float(pq.lower), (int)pi.lower, __uint_as_float(pq.upper), (int)pi.upper, best_q, best_idx);
        pq = halves32(__float_as_uint(best_q));
        pi = halves32((uint32_t)best_idx);
        better(__uint_as_float(pq.lower), (int)pi.lower, __uint_as_float(pq.upper), (int)pi.upper, best_q, best_idx);
    }
}

// The unroll's per-slot reductions below go through LDS shuffles instead: they cost the wave a
// wait but no vector issue slots, which it shares with a compute wave; and with their cost off
// the SIMD the online and the target workgroup of a tile keep the same pace, so the second of them
// to read an observation line still finds it in L2.
//
// Maximum of the row's available Q values (0 when nothing is available).
template <int AB>
__device__ __forceinline__ float masked_max16(const f32x4 (&qv)[AB], uint32_t slots)
{
    float m = -__builtin_inff();
#pragma unroll
    for (int ab = 0; ab < AB; ++ab)
#pragma unroll
        for (int r = 0; r < 4; ++r) m = fmaxf(m, ((slots >> (4 * ab + r)) & 1u) ? qv[ab][r] : -__builtin_inff());
    m = fmaxf(m, __shfl_xor(m, 16));
    m = fmaxf(m, __shfl_xor(m, 32));
    return m == -__builtin_inff() ? 0.0f : m;
}

// Q value of action u of this lane's row (one of the four lanes has it; they are summed).
template <int AB>
__device__ __forceinline__ float pick_action_value16(const f32x4 (&qv)[AB], int u, int q)
{
    float v = 0.0f;
#pragma unroll
    for (int ab = 0; ab < AB; ++ab)
#pragma unroll
        for (int r = 0; r < 4; ++r) v = (16 * ab + 4 * q + r == u) ? qv[ab][r] : v;
    v += __shfl_xor(v, 16);
    return v + __shfl_xor(v, 32);
}

template <int AB>
__device__ __forceinline__ void store_q_row16(float *__restrict__ q_row, const f32x4 (&qv)[AB], int A, int q)
{
#pragma unroll
    for (int ab = 0; ab < AB; ++ab)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int a = 16 * ab + 4 * q + r;
            if (a < A) q_row[a] = qv[ab][r];
        }
}

}  // namespace marl
