// Wave-level building blocks: one wavefront evaluates the network for a tile of
// 32 (env, agent) rows with 32x32x16 bf16 MFMAs.  Weights are the A operand
// (32 output features x 16 k), activations the B operand (16 k x 32 rows), so an
// accumulator holds [32 features x 32 rows] and lane l owns row l % 32.  Because
// both lanes l and l + 32 of a row keep whole groups of four consecutive
// features, a result is converted to the next layer's B operand in registers
// (the weight fragments are stored in the matching k order).
//
// P = 1: bf16 weights, activations rounded to bf16, fp32 accumulation.
// P = 2: fp32 weights and activations, each split into a bf16 high part and the
//        bf16 of the remainder; products hi*hi + hi*lo + lo*hi in fp32
//        accumulators (error about 2^-16 relative per product).
#pragma once
#include "device_math.h"
#include "qnet_internal.h"

namespace marl {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int P> struct Frag;
template <> struct Frag<1> { bf16x8 hi; };
template <> struct Frag<2> { bf16x8 hi, lo; };

template <int P>
__device__ __forceinline__ Frag<P> to_frag(const float (&v)[8])
{
    Frag<P> f;
#pragma unroll
    for (int i = 0; i < 8; ++i) f.hi[i] = (__bf16)v[i];
    if constexpr (P == 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) f.lo[i] = (__bf16)(v[i] - (float)f.hi[i]);
    }
    return f;
}

// Values r = 8c .. 8c+7 of an accumulator block become k-chunk 2*block + c of the next operand.
template <int P>
__device__ __forceinline__ Frag<P> frag_of_half(const f32x16 &acc, int c)
{
    float v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = c ? acc[8 + i] : acc[i];
    return to_frag<P>(v);
}

// acc += Wfrag * b ; `a` points at this lane's 16 bytes of plane 0 of the fragment.
template <int P>
__device__ __forceinline__ void mma(f32x16 &acc, const bf16x8 *a, const Frag<P> &b)
{
    const bf16x8 ah = a[0];
    if constexpr (P == 2) {
        const bf16x8 al = a[64];
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, b.hi, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b.lo, acc, 0, 0, 0);
    }
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ah, b.hi, acc, 0, 0, 0);
}

// A weight fragment held in registers so that it can feed several column blocks.
template <int P> struct WFrag;
template <> struct WFrag<1> { bf16x8 hi; };
template <> struct WFrag<2> { bf16x8 hi, lo; };

template <int P>
__device__ __forceinline__ WFrag<P> load_wfrag(const bf16x8 *a)
{
    WFrag<P> w;
    w.hi = a[0];
    if constexpr (P == 2) w.lo = a[64];
    return w;
}

template <int P>
__device__ __forceinline__ void mma(f32x16 &acc, const WFrag<P> &w, const Frag<P> &b)
{
    if constexpr (P == 2) {
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w.lo, b.hi, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w.hi, b.lo, acc, 0, 0, 0);
    }
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w.hi, b.hi, acc, 0, 0, 0);
}

// Feature held in accumulator slot r of block `blk` by a lane of half g: 32 blk + 8 (r / 4) + 4 g + r % 4.
// The four slots 4j .. 4j+3 are consecutive features, so per-feature tables load as float4.
__device__ __forceinline__ f32x16 load_feature_block(const float *table, int blk, int g)
{
    f32x16 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const f32x4 t = *reinterpret_cast<const f32x4 *>(table + 32 * blk + 8 * j + 4 * g);
        v[4 * j + 0] = t[0]; v[4 * j + 1] = t[1]; v[4 * j + 2] = t[2]; v[4 * j + 3] = t[3];
    }
    return v;
}

__device__ __forceinline__ void store_feature_block(float *dst, int blk, int g, const f32x16 &v)
{
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        f32x4 t = {v[4 * j + 0], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]};
        *reinterpret_cast<f32x4 *>(dst + 32 * blk + 8 * j + 4 * g) = t;
    }
}

// Eight observation values 16 kc + 8 g + (0..7) of one row.  Branch-free on purpose: a guarded
// load makes the compiler wait for each one separately.  Positions at or beyond D are read from
// clamped (in-row) addresses instead; the weight fragments are zero there, so whatever finite
// value arrives contributes nothing.  `row` must always point at a readable row.
__device__ __forceinline__ void load_obs_chunk(const float *__restrict__ row, int D, bool vec4, int kc, int g, float (&v)[8])
{
    const int k0 = 16 * kc + 8 * g;
    if (vec4) {   // D % 4 == 0 and the row is 16-byte aligned
        const f32x4 a = *reinterpret_cast<const f32x4 *>(row + min(k0, D - 4));
        const f32x4 b = *reinterpret_cast<const f32x4 *>(row + min(k0 + 4, D - 4));
        v[0] = a[0]; v[1] = a[1]; v[2] = a[2]; v[3] = a[3];
        v[4] = b[0]; v[5] = b[1]; v[6] = b[2]; v[7] = b[3];
    } else {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = row[min(k0 + i, D - 1)];
    }
}

// h' = (1 - z) * n + z * h on one block of 16 slots.
__device__ __forceinline__ f32x16 gru_blend(const f32x16 &ar, const f32x16 &az, const f32x16 &ain, const f32x16 &ahn,
                                            const f32x16 &h)
{
    f32x16 out;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const float rr = sigmoidf_fast(ar[r]), zz = sigmoidf_fast(az[r]);
        const float nn = tanhf_fast(ain[r] + rr * ahn[r]);
        out[r] = fmaf(zz, h[r] - nn, nn);            // (1 - z) n + z h
    }
    return out;
}

// Availability of the actions this lane holds, in two steps so that the loads can be issued
// long before the mask is needed.
//
// issue_avail_loads: the four actions of one accumulator group (32 mb + 8 j + 4 g + 0..3) are
// adjacent bytes and are fetched with one, possibly unaligned, 32-bit load whose address is
// clamped into the row; every load is unconditional and independent.  avail_row must point at a
// readable row of A >= 4 bytes (rows with fewer actions use avail_mask_small).
template <int MB2>
__device__ __forceinline__ void issue_avail_loads(const uint8_t *__restrict__ avail_row, int A, int lane,
                                                  uint32_t (&raw)[MB2 * 4])
{
    const int g = lane >> 5;
#pragma unroll
    for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int base = min(32 * mb + 8 * j + 4 * g, A - 4);
            __builtin_memcpy(&raw[mb * 4 + j], avail_row + base, 4);
        }
}

// Bit 16 mb + r of the result is set when action 32 mb + 8 (r / 4) + 4 g + r % 4 exists and is
// available.
template <int MB2>
__device__ __forceinline__ uint32_t avail_mask_from_raw(const uint32_t (&raw)[MB2 * 4], int A, int lane, bool valid)
{
    const int g = lane >> 5;
    uint32_t mask = 0;
#pragma unroll
    for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int a0 = 32 * mb + 8 * j + 4 * g;
            const int skip = a0 - min(a0, A - 4);                  // bytes of the word that precede a0
            const uint32_t w = skip < 4 ? raw[mb * 4 + j] >> (8 * skip) : 0u;
#pragma unroll
            for (int i = 0; i < 4; ++i) mask |= ((w >> (8 * i)) & 0xFFu) ? (1u << (16 * mb + 4 * j + i)) : 0u;
        }
    return valid ? mask : 0u;
}

// Rows with fewer than four actions: they all sit in the first group of the lower half-wave.
__device__ __forceinline__ uint32_t avail_mask_small(const uint8_t *__restrict__ avail_row, int A, int lane, bool valid)
{
    uint32_t mask = 0;
#pragma unroll
    for (int i = 0; i < 3; ++i) {
        const uint32_t v = avail_row[min(i, A - 1)];
        mask |= (i < A && v) ? (1u << i) : 0u;
    }
    return (valid && lane < 32) ? mask : 0u;
}

// A row's Q values are split over lanes l and l ^ 32.  Masked maximum with the lowest index on ties.
// idx = -1 and best_q = 0 when nothing is available.
template <int MB2>
__device__ __forceinline__ void masked_argmax_slots(const f32x16 (&q)[MB2], uint32_t slots, int lane, float &best_q,
                                                    int &best_idx)
{
    const int g = lane >> 5;
    best_q = 0.0f; best_idx = -1;
#pragma unroll
    for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int a = 32 * mb + 8 * (r / 4) + 4 * g + (r % 4);
            const bool ok = (slots >> (16 * mb + r)) & 1u;
            if (ok && (best_idx < 0 || q[mb][r] > best_q)) { best_q = q[mb][r]; best_idx = a; }
        }
    const float oq = __shfl_xor(best_q, 32);
    const int oi = __shfl_xor(best_idx, 32);
    if (oi >= 0 && (best_idx < 0 || oq > best_q || (oq == best_q && oi < best_idx))) { best_q = oq; best_idx = oi; }
}

// Maximum of the row's available Q values (0 when nothing is available); no index.
template <int MB2>
__device__ __forceinline__ float masked_max_slots(const f32x16 (&q)[MB2], uint32_t slots)
{
    float m = -__builtin_inff();
#pragma unroll
    for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) m = fmaxf(m, ((slots >> (16 * mb + r)) & 1u) ? q[mb][r] : -__builtin_inff());
    m = fmaxf(m, __shfl_xor(m, 32));
    return m == -__builtin_inff() ? 0.0f : m;
}

// Availability bits of the whole row (bit a = action a) from the two lanes' slot masks.
template <int MB2>
__device__ __forceinline__ uint64_t row_avail_bits(uint32_t slots, int lane)
{
    const int g = lane >> 5;
    uint64_t bits = 0;
#pragma unroll
    for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int a = 32 * mb + 8 * (r / 4) + 4 * g + (r % 4);
            if ((slots >> (16 * mb + r)) & 1u) bits |= 1ull << a;
        }
    const uint32_t olo = __shfl_xor((uint32_t)bits, 32), ohi = __shfl_xor((uint32_t)(bits >> 32), 32);
    return bits | ((uint64_t)ohi << 32) | olo;
}

// Q value of action u of this lane's row (the owner lane has it; the pair is summed).
template <int MB2>
__device__ __forceinline__ float pick_action_value(const f32x16 (&q)[MB2], int u, int lane)
{
    const int g = lane >> 5;
    float v = 0.0f;
#pragma unroll
    for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int a = 32 * mb + 8 * (r / 4) + 4 * g + (r % 4);
            v = (a == u) ? q[mb][r] : v;
        }
    return v + __shfl_xor(v, 32);
}

// Store this lane's share of a row of Q ([A] floats at q_row).
template <int MB2>
__device__ __forceinline__ void store_q_row(float *__restrict__ q_row, const f32x16 (&q)[MB2], int A, int lane)
{
    const int g = lane >> 5;
#pragma unroll
    for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int a = 32 * mb + 8 * (r / 4) + 4 * g + (r % 4);
            if (a < A) q_row[a] = q[mb][r];
        }
}

}  // namespace marl
