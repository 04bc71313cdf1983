// Device-side scalar helpers shared by the kernels of this library: gate
// non-linearities of the GRU cell, the SplitMix64 counter generator used by the
// epsilon-greedy rule of the decision step, and the per-row action choice.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace marl {

// Gate non-linearities on the hardware exp2 / reciprocal units (about 1 ulp each).
// exp2 overflowing to +inf gives rcp = 0 and underflowing to 0 gives rcp(1) = 1, so both
// functions saturate cleanly for large |v|.
constexpr float kLog2e = 1.4426950408889634f;

__device__ __forceinline__ float sigmoidf_fast(float v)
{
    return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-kLog2e * v));
}

// tanh(v) = 1 - 2 / (1 + e^{2v}); absolute error about 1e-7.
__device__ __forceinline__ float tanhf_fast(float v)
{
    return fmaf(-2.0f, __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(2.0f * kLog2e * v)), 1.0f);
}

// SplitMix64 (Steele, Lea, Flood 2014): state += golden gamma, then the 64-bit finaliser.
constexpr uint64_t kGolden = 0x9E3779B97F4A7C15ull;

__device__ __forceinline__ uint64_t splitmix_out(uint64_t v)
{
    v += kGolden;
    v ^= v >> 30; v *= 0xBF58476D1CE4E5B9ull;
    v ^= v >> 27; v *= 0x94D049BB133111EBull;
    v ^= v >> 31;
    return v;
}

// Two draws for (seed, env, agent, step): the key chains the four words through the generator.
__device__ __forceinline__ void rng_draw(uint64_t seed, uint32_t e, uint32_t n, uint32_t t,
                                         uint64_t &r1, uint64_t &r2)
{
    uint64_t k = splitmix_out(splitmix_out(splitmix_out(splitmix_out(seed) ^ e) ^ n) ^ t);
    r1 = splitmix_out(k);
    r2 = splitmix_out(k + kGolden);
}

// Index of the j-th set bit of bits (j counted from 0, j < popcount(bits)): a binary search on
// the population counts of the lower halves, the same number of steps for every lane.
__device__ __forceinline__ int nth_set_bit(uint64_t bits, uint32_t j)
{
    uint32_t word = (uint32_t)bits;
    int base = 0;
    const uint32_t below = (uint32_t)__popc(word);
    if (j >= below) { j -= below; word = (uint32_t)(bits >> 32); base = 32; }
#pragma unroll
    for (int half = 16; half >= 1; half >>= 1) {
        const uint32_t low = word & ((1u << half) - 1u);
        const uint32_t cnt = (uint32_t)__popc(low);
        const bool up = j >= cnt;
        j = up ? j - cnt : j;
        word = up ? word >> half : low;
        base = up ? base + half : base;
    }
    return base;
}

// The uniform draw and the raw second draw for (seed, env, agent, step); explore when u < epsilon.
struct ExploreDraw { float u; uint32_t pick_bits; };
__device__ __forceinline__ ExploreDraw explore_draw(uint64_t seed, uint32_t e, uint32_t n, uint32_t t)
{
    uint64_t r1, r2;
    rng_draw(seed, e, n, t, r1, r2);
    return {(float)(uint32_t)(r1 >> 40) * (1.0f / 16777216.0f), (uint32_t)(r2 >> 32)};
}

// Epsilon-greedy over the available actions of one (env, agent) row, given the
// greedy action and the availability bits (bit a of avail_bits = action a usable).
__device__ __forceinline__ int eps_greedy_pick(int greedy, uint64_t avail_bits, float epsilon,
                                               uint64_t seed, uint32_t e, uint32_t n, uint32_t t)
{
    const ExploreDraw d = explore_draw(seed, e, n, t);
    if (!(d.u < epsilon)) return greedy;
    const uint32_t c = (uint32_t)__popcll(avail_bits);
    if (c == 0) return 0;
    const uint32_t j = (uint32_t)(((uint64_t)d.pick_bits * (uint64_t)c) >> 32);      // uniform over 0 .. c-1
    return nth_set_bit(avail_bits, j);
}

}  // namespace marl
