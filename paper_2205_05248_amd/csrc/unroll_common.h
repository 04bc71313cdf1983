// Pieces shared by the unroll kernels: the LDS-only workgroup barrier and the record layout of
// the input half of the GRU gates (written by the projection, consumed by the recurrence).
#pragma once
#include "mfma_tile.h"

namespace marl {

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every global
// load and store of the wave, which would expose the latency of the prefetches that are meant
// to stay in flight across slots.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// Scratch written by the input projection and read by the recurrent kernel: one record per
// (row tile, slot) holding, for each gate and hidden block, the 32x32 accumulator of that block in
// lane order, so that every wave-wide access is contiguous.
//   fp32 networks: fp32 values, [3 gates][H/32][4][64 lanes][4]   (slots 4j..4j+3 of lane l at [j][l])
//   bf16 networks: bf16 values, [3 gates][H/32][2][64 lanes][8]   (slots 8p..8p+7 of lane l at [p][l])
// bf16 halves the traffic of the two kernels, which are bound by it; the rounding (2^-9 relative on
// pre-activations of order one) stays well inside that mode's tolerance.
template <int P> struct GiLayout {
    static constexpr bool kBf16 = P == 1;
    static constexpr int kBlockBytes = kBf16 ? 2048 : 4096;            // one gate, one hidden block
    static constexpr int block_vecs() { return kBlockBytes / 16; }
};

template <int P>
__device__ __forceinline__ void store_gi_block(char *__restrict__ dst, int lane, const f32x16 &v)
{
    if constexpr (GiLayout<P>::kBf16) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            bf16x8 t;
#pragma unroll
            for (int i = 0; i < 8; ++i) t[i] = (__bf16)v[8 * p + i];
            *reinterpret_cast<bf16x8 *>(dst + p * 1024 + lane * 16) = t;
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const f32x4 t = {v[4 * j + 0], v[4 * j + 1], v[4 * j + 2], v[4 * j + 3]};
            *reinterpret_cast<f32x4 *>(dst + j * 1024 + lane * 16) = t;
        }
    }
}

// The same block read back from an LDS copy of the record.
template <int P>
__device__ __forceinline__ f32x16 load_gi_block(const char *src, int lane)
{
    f32x16 v;
    if constexpr (GiLayout<P>::kBf16) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const bf16x8 t = *reinterpret_cast<const bf16x8 *>(src + p * 1024 + lane * 16);
#pragma unroll
            for (int i = 0; i < 8; ++i) v[8 * p + i] = (float)t[i];
        }
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const f32x4 t = *reinterpret_cast<const f32x4 *>(src + j * 1024 + lane * 16);
            v[4 * j + 0] = t[0]; v[4 * j + 1] = t[1]; v[4 * j + 2] = t[2]; v[4 * j + 3] = t[3];
        }
    }
    return v;
}

}  // namespace marl
