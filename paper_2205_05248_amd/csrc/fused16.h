// Shape and LDS layout shared by the fused kernels on tiles of 16 rows (unroll_fused.hip,
// act_fused.hip): which wavefront plays which role, what stays resident where, and the byte
// offsets of the LDS buffers.
#pragma once
#include <atomic>

#include "mfma16_tile.h"
#include "unroll_common.h"

namespace marl {

// Host: the runtime has to be told, once per kernel and device, that launches of it may ask for
// more than 64 KB of dynamic LDS.  The current device is the one the launch will go to.
template <auto Kernel>
hipError_t allow_large_lds(int bytes)
{
    static std::atomic<uint64_t> done{0};            // one bit per device id
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    const uint64_t bit = 1ull << (dev & 63);
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    err = hipFuncSetAttribute(reinterpret_cast<const void *>(Kernel), hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (err == hipSuccess) done.fetch_or(bit, std::memory_order_release);
    return err;
}

constexpr int kFusedLead = 3;         // steps before slot 0 enters the recurrence
constexpr int kLdsLimit = 160 * 1024;
constexpr int kRawBuffer = 0x00020000;       // descriptor word 3: untyped 32-bit data, no swizzle, offsets checked against the size

template <int H, int P> struct Fused16 {
    static constexpr int FBK = H / 16;                 // feature blocks of the hidden layer
    static constexpr int KS = H / 32;                  // k-steps over the hidden layer
    static constexpr int NC = 4;                       // compute waves
    static constexpr int NBC = FBK / NC;               // feature blocks per compute wave (2 or 1)
    static constexpr int NF = 2;                       // fc1 waves
    static constexpr int kEpilogue = NC, kLoader = NC + 1, kFc1 = NC + 2, kWaves = NC + 2 + NF;
    static constexpr int NBF = FBK / NF;               // fc1 feature blocks per fc1 wave
    static constexpr int kKs1Max = 10 / P;             // observation k-steps: W1 fragments of an fc1 wave within 160 registers (H = 128), 80 (H = 64)
    static constexpr int kFrag = P * 1024;             // bytes of one fragment (all planes)
    // LDS layout (byte offsets)
    static constexpr int oWih = 0;                                  // [3 FBK][KS][P][64] bf16x8
    static constexpr int oH = oWih + 3 * FBK * KS * kFrag;          // [2][KS][P][64] bf16x8
    static constexpr int oX = oH + 2 * KS * kFrag;                  // [2][KS][P][64] bf16x8
    static constexpr int oGBias = oX + 2 * KS * kFrag;              // [3 H] floats: b_ir + b_hr, b_iz + b_hz, b_in
    static constexpr int oB2 = oGBias + 3 * H * 4;                  // [64] floats
    static constexpr int oObs = oB2 + 256;                          // [2][ks1][P][64] bf16x8
    static constexpr size_t lds_bytes(int ks1) { return (size_t)oObs + (size_t)2 * ks1 * kFrag; }
    // decision step only, after the observations: the incoming hidden state as operand fragments
    // [2][KS][P][64] bf16x8, then in fp32 by feature block [2][FBK][64] float4
    static constexpr size_t hin_offset(int ks1) { return lds_bytes(ks1); }
    static constexpr size_t hf_offset(int ks1) { return hin_offset(ks1) + (size_t)2 * KS * kFrag; }
    // then what the loader and the epilogue hand each other about the choice of action: the
    // availability slots of every lane [2][64] words, and per row of the last eight items the
    // availability bits and step number [8][16] x 12 bytes and the greedy action [8][16] bytes
    static constexpr size_t slots_offset(int ks1) { return hf_offset(ks1) + (size_t)2 * FBK * 1024; }
    static constexpr size_t choice_offset(int ks1) { return slots_offset(ks1) + 512; }
    static constexpr size_t greedy_offset(int ks1) { return choice_offset(ks1) + 8 * 16 * 12; }
    static constexpr size_t lds_bytes_act(int ks1) { return greedy_offset(ks1) + 8 * 16; }
};

constexpr int fused_threads(int) { return 64 * (4 + 2 + 2); }

}  // namespace marl
