// Fused unroll + TD kernel for gfx950: one workgroup walks the T+1 slots of one tile of 32
// (episode, agent) rows for one network and never writes an intermediate to global memory.
//
// The work of a slot is cut into pipeline stages that run concurrently on different wavefronts,
// each stage working on a different slot, and meet at ONE LDS-only barrier per slot.  In the step
// in which the recurrence handles slot s:
//
//   loader wave    issues the global loads of the observations of slot s+4 (one row per lane
//                  pair, the k order of an MFMA B operand) and writes those of slot s+3, loaded
//                  during the previous step, to LDS as bf16 operand fragments;
//   fc1 wave       x = ReLU(W1 o + b1[agent]) for slot s+2: observation fragments from LDS, W1
//                  fragments streamed from L2 through a ring of registers; x goes to LDS as the
//                  next operand;
//   gates wave     W_ih x + b for slot s+1 (all three gates, every hidden block), W_ih streamed
//                  the same way; results go to LDS in the block form the recurrence reads;
//   compute waves  slot s of the recurrence (recurrent_roles.h);
//   epilogue wave  fc2 / TD step of slot s-1 (recurrent_roles.h).
//
// Only the recurrence is a dependent chain; every other stage is throughput work that hides
// under it.  Global traffic per slot and tile: the observations once, the TD inputs and outputs,
// and the W1 / W_ih fragments (from L2: every workgroup of a network streams the same ones).
//
// Every LDS buffer is double-buffered on the parity of the slot it holds; a buffer written in
// step s was last read in step s-1 and is first read in step s+1.
#include <hip/hip_runtime.h>

#include "recurrent_roles.h"

namespace marl {

constexpr int kFusedMaxKc1 = 24;      // observation k-steps the loader can hold in registers
constexpr int kFusedLead = 4;         // steps before slot 0 enters the recurrence
constexpr int kLdsLimit = 160 * 1024;

constexpr int fused_min(int a, int b) { return a < b ? a : b; }

template <int H, int P> struct FusedShape {
    static constexpr int MB = H / 32, KCH = H / 16;
    static constexpr int kEpilogue = MB, kLoader = MB + 1, kFc1 = MB + 2, kGates = MB + 3, kWaves = MB + 4;
    static constexpr int kGiBytes = 3 * MB * GiLayout<P>::kBlockBytes;
    static constexpr int kFragBytes = P * 1024;
    static constexpr int kHBytes = KCH * kFragBytes;
    // fc1 wave: k-steps of W1 (MB fragments each) in flight; 24 planes = 96 registers
    static constexpr int kRingKc = 24 / (MB * P);
    // gates wave: fragments per slot, and how many are in flight (divides the former)
    static constexpr int kGateFrags = 3 * MB * KCH;
    static constexpr int kGateRing = fused_min(24 / P, kGateFrags);
    static_assert(kGateFrags % kGateRing == 0, "the ring must map every fragment to a fixed register");
    // LDS layout (byte offsets)
    static constexpr int oGi = 0;                              // [2][kGiBytes]
    static constexpr int oH = oGi + 2 * kGiBytes;              // [2][KCH][P][64] bf16x8
    static constexpr int oX = oH + 2 * kHBytes;                // [2][KCH][P][64] bf16x8
    static constexpr int oBias1 = oX + 2 * kHBytes;            // [MB][4][64] float4: fc1 bias of the tile's rows, accumulator form
    static constexpr int oGBias = oBias1 + MB * 4096;          // [3 MB][32] floats: gate biases by block
    static constexpr int oB2 = oGBias + 3 * MB * 128;          // [64] floats
    static constexpr int oObs = oB2 + 256;                     // [2][kc1][P][64] bf16x8
    static constexpr size_t lds_bytes(int kc1) { return (size_t)oObs + (size_t)2 * kc1 * kFragBytes; }
};

constexpr int fused_threads(int H) { return 64 * (H / 32 + 4); }

template <int H, int P, int MB2, bool QALL>
__global__ __launch_bounds__(fused_threads(H), 2) void unroll_fused_kernel(
    NetFrags online, NetFrags target, int two_nets, int B, int T, const float *__restrict__ obs,
    const uint8_t *__restrict__ avail, const int32_t *__restrict__ actions, const float *__restrict__ reward,
    const uint8_t *__restrict__ terminated, const uint8_t *__restrict__ filled, float gamma,
    float *__restrict__ q_taken, float *__restrict__ next_max, float *__restrict__ td_target, float *__restrict__ q_all)
{
    using Sh = FusedShape<H, P>;
    constexpr int MB = Sh::MB, KCH = Sh::KCH, LEAD = kFusedLead;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    typedef bf16x8 (*FragBuf)[KCH][P][64];
    const FragBuf h_lds = reinterpret_cast<FragBuf>(lds + Sh::oH);
    const FragBuf x_lds = reinterpret_cast<FragBuf>(lds + Sh::oX);
    bf16x8 *const obuf = reinterpret_cast<bf16x8 *>(lds + Sh::oObs);        // [(slot & 1) kc1 + kc][P][64]

    const bool is_target = blockIdx.y == 1;
    const NetFrags &net = is_target ? target : online;
    const int lane = threadIdx.x & 63, g = lane >> 5, col = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rt = blockIdx.x;
    const int N = net.N, D = net.D, kc1 = net.kc1, S = T + 1;
    // Steps run s = -LEAD .. T+1, one barrier at the end of each: T + 2 + LEAD barriers per wave.

    if (wave < MB) {
        compute_role<H, P>(net, wave, lane, T, LEAD, lds + Sh::oGi, h_lds);
    } else if (wave == Sh::kEpilogue) {
        const TdArrays td{avail, actions, reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all};
        epilogue_role<H, P, MB2, QALL>(net, td, !is_target, is_target || !two_nets, rt, lane, B, T, LEAD, h_lds,
                                       reinterpret_cast<float *>(lds + Sh::oB2));
    } else if (wave == Sh::kLoader) {
        // ---------------------------------------------------------------- loader wave
        const int row = rt * 32 + col;
        const bool valid = row < B * N;                    // rows past the end read row 0; their results are dropped
        const int b = valid ? row / N : 0, n = valid ? row % N : 0;
        const float *base = obs + ((size_t)b * S * N + n) * D + 8 * g;     // this lane's half of k-step 0, slot 0
        const size_t slot_stride = (size_t)N * D;
        // k-steps that lie wholly inside the row are fetched as two 16-byte loads at constant
        // offsets from one address (only 4-byte alignment is assumed, which every row has); the
        // last, partial k-step is fetched element by element from clamped positions, whose
        // weights are zero.
        const int kc_full = D / 16;
        int tail_off[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) tail_off[i] = min(16 * kc_full + 8 * g + i, D - 1) - 8 * g;
        float stage[kFusedMaxKc1][8];
        for (int s = -LEAD; s <= T + 1; ++s) {
            const int ws = s + 3, ls = s + 4;
            if (ws >= 0 && ws <= T) {
                bf16x8 *dst = obuf + (size_t)((ws & 1) * kc1) * P * 64 + lane;
#pragma unroll
                for (int kc = 0; kc < kFusedMaxKc1; ++kc)
                    if (kc < kc1) {
                        const Frag<P> f = to_frag<P>(stage[kc]);
                        dst[(kc * P) * 64] = f.hi;
                        if constexpr (P == 2) dst[(kc * P + 1) * 64] = f.lo;
                    }
            }
            if (ls >= 0 && ls <= T) {
                const float *r = base + (size_t)ls * slot_stride;
#pragma unroll
                for (int kc = 0; kc < kFusedMaxKc1; ++kc) {
                    if (kc < kc_full) {
                        f32x4 lo4, hi4;
                        __builtin_memcpy(&lo4, r + 16 * kc, 16);
                        __builtin_memcpy(&hi4, r + 16 * kc + 4, 16);
#pragma unroll
                        for (int i = 0; i < 4; ++i) { stage[kc][i] = lo4[i]; stage[kc][4 + i] = hi4[i]; }
                    } else if (kc < kc1) {
#pragma unroll
                        for (int i = 0; i < 8; ++i) stage[kc][i] = r[tail_off[i]];
                    }
                }
            }
            lds_barrier();
        }
    } else if (wave == Sh::kFc1) {
        // ---------------------------------------------------------------- fc1 wave
        constexpr int RK = Sh::kRingKc;
        const int row = rt * 32 + col;
        const int n = row < B * N ? row % N : 0;
        f32x4 *const btab = reinterpret_cast<f32x4 *>(lds + Sh::oBias1);     // private to this wave
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                btab[(mb * 4 + j) * 64 + lane] = *reinterpret_cast<const f32x4 *>(net.bias1 + (size_t)n * H + 32 * mb + 8 * j + 4 * g);

        // W1 fragments, [k-step][feature block]; the same kc1 k-steps every slot, so the ring just
        // keeps running RK-1 k-steps ahead across slot boundaries.
        const bf16x8 *w1 = net.w1_seq + lane;
        WFrag<P> ring[RK][MB];
        int ppos = 0;
        auto prefetch = [&](int slot) {
#pragma unroll
            for (int mb = 0; mb < MB; ++mb) ring[slot][mb] = load_wfrag<P>(w1 + (size_t)((ppos * MB + mb) * P) * 64);
            if (++ppos == kc1) ppos = 0;
        };
        auto obs_frag = [&](int slot, int kc) {
            const bf16x8 *src = obuf + (size_t)(((slot & 1) * kc1 + kc) * P) * 64 + lane;
            Frag<P> f;
            f.hi = src[0];
            if constexpr (P == 2) f.lo = src[64];
            return f;
        };
#pragma unroll
        for (int r = 0; r < RK - 1; ++r) prefetch(r);
        f32x16 acc[MB];
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int i = 0; i < 16; ++i) acc[mb][i] = 0.0f;
        for (int s = -LEAD; s < -2; ++s) lds_barrier();

        int slot = 0, kpos = 0;                      // step s handles slot s + 2
        // observation fragments are read from LDS OB k-steps ahead of their MFMAs (LDS latency);
        // positions past the slot's last k-step re-read it and are dropped at the slot change
        constexpr int OB = 3;
        Frag<P> bq[OB];
#pragma unroll
        for (int i = 0; i < OB; ++i) bq[i] = obs_frag(0, min(i, kc1 - 1));
        const long total = (long)(T + 1) * kc1;      // k-steps of the whole episode
        for (long it = 0; it < total; it += RK) {
#pragma unroll
            for (int r = 0; r < RK; ++r) {
                prefetch((r + RK - 1) % RK);         // past the end: harmless reloads of the first k-steps
                if (it + r >= total) continue;
                const Frag<P> bnext = obs_frag(slot, min(kpos + OB, kc1 - 1));
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) mma<P>(acc[mb], ring[r][mb], bq[0]);
#pragma unroll
                for (int i = 0; i + 1 < OB; ++i) bq[i] = bq[i + 1];
                bq[OB - 1] = bnext;
                if (++kpos == kc1) {
                    // bias, ReLU, and hand x over as the next operand
#pragma unroll
                    for (int mb = 0; mb < MB; ++mb) {
                        f32x16 v;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            const f32x4 t = btab[(mb * 4 + j) * 64 + lane];
#pragma unroll
                            for (int i = 0; i < 4; ++i) v[4 * j + i] = fmaxf(acc[mb][4 * j + i] + t[i], 0.0f);
                        }
#pragma unroll
                        for (int c = 0; c < 2; ++c) {
                            const Frag<P> f = frag_of_half<P>(v, c);
                            x_lds[slot & 1][2 * mb + c][0][lane] = f.hi;
                            if constexpr (P == 2) x_lds[slot & 1][2 * mb + c][1][lane] = f.lo;
                        }
#pragma unroll
                        for (int i = 0; i < 16; ++i) acc[mb][i] = 0.0f;
                    }
                    lds_barrier();
                    kpos = 0;
                    ++slot;
                    if (slot <= T) {
#pragma unroll
                        for (int i = 0; i < OB; ++i) bq[i] = obs_frag(slot, min(i, kc1 - 1));
                    }
                }
            }
        }
        for (int s = T - 1; s <= T + 1; ++s) lds_barrier();
    } else {
        // ---------------------------------------------------------------- gates wave
        constexpr int NF = Sh::kGateFrags, RG = Sh::kGateRing;
        constexpr bool RESIDENT = RG == NF;          // the whole matrix fits the ring: load it once
        float *const gb = reinterpret_cast<float *>(lds + Sh::oGBias);       // private to this wave
        for (int i = lane; i < 3 * H; i += 64) {
            const int gate = i / H, j = i % H;       // block gate * MB + j / 32, feature j % 32
            const float *src = gate == 0 ? net.bias_r : gate == 1 ? net.bias_z : net.bias_in;
            gb[i] = src[j];
        }
        // W_ih fragments in order of use: [pass][k-step][block of the pass], three blocks per pass
        // The fragments are read in sequence through one running byte offset.  It is kept opaque to
        // the compiler, which would otherwise precompute one address per fragment of the slot and
        // keep (spill) all of them across the slot loop.
        const char *wg = reinterpret_cast<const char *>(net.wih_seq);
        uint32_t woff = lane * 16;
        auto load_next = [&](bool wrap) {
            WFrag<P> w;
            w.hi = *reinterpret_cast<const bf16x8 *>(wg + woff);
            if constexpr (P == 2) w.lo = *reinterpret_cast<const bf16x8 *>(wg + woff + 1024);
            woff = wrap ? lane * 16 : woff + P * 1024;
            asm volatile("" : "+v"(woff));
            return w;
        };
        WFrag<P> ring[RG];
#pragma unroll
        for (int f = 0; f < (RESIDENT ? RG : RG - 1); ++f) ring[f] = load_next(false);
        for (int s = -LEAD; s < -1; ++s) lds_barrier();

        for (int slot = 0; slot <= T; ++slot) {      // step s handles slot s + 1
            const int buf = slot & 1;
            Frag<P> x[KCH];                          // the slot's fc1 output, read once
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) {
                x[kc].hi = x_lds[buf][kc][0][lane];
                if constexpr (P == 2) x[kc].lo = x_lds[buf][kc][1][lane];
            }
            char *gi_dst = lds + Sh::oGi + buf * Sh::kGiBytes;
#pragma unroll
            for (int pass = 0; pass < MB; ++pass) {
                f32x16 acc[3];
#pragma unroll
                for (int b = 0; b < 3; ++b) acc[b] = load_feature_block(gb, 3 * pass + b, g);
#pragma unroll
                for (int kc = 0; kc < KCH; ++kc) {
#pragma unroll
                    for (int b = 0; b < 3; ++b) {
                        const int f = (pass * KCH + kc) * 3 + b;
                        if constexpr (!RESIDENT) {
                            ring[(f + RG - 1) % RG] = load_next((f + RG - 1) % NF == NF - 1);
                        }
                        mma<P>(acc[b], ring[f % RG], x[kc]);
                    }
                }
#pragma unroll
                for (int b = 0; b < 3; ++b)
                    store_gi_block<P>(gi_dst + (3 * pass + b) * GiLayout<P>::kBlockBytes, lane, acc[b]);
            }
            lds_barrier();
        }
        for (int s = T; s <= T + 1; ++s) lds_barrier();
    }
}

// ------------------------------------------------------------------------------------------ host side
namespace {

template <int H, int P>
hipError_t fused_dispatch(const NetFrags &online, const NetFrags &target, bool two_nets, int B, int T,
                          const float *obs, const uint8_t *avail, const int32_t *actions, const float *reward,
                          const uint8_t *terminated, const uint8_t *filled, float gamma, float *q_taken,
                          float *next_max, float *td_target, float *q_all, hipStream_t stream)
{
    using Sh = FusedShape<H, P>;
    const int tiles = (B * online.N + 31) / 32;
    const dim3 grid((unsigned)tiles, two_nets ? 2u : 1u), block(64 * Sh::kWaves);
    const size_t lds = Sh::lds_bytes(online.kc1);
    const int two = two_nets ? 1 : 0;
#define MARL_FUSED(MB, QA)                                                                                          \
    do {                                                                                                            \
        auto kernel = unroll_fused_kernel<H, P, MB, QA>;                                                            \
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),                               \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                 \
        if (err != hipSuccess) return err;                                                                          \
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, online, target, two, B, T, obs, avail, actions,        \
                           reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all);                 \
    } while (0)
    if (online.mb2 == 1) { if (q_all) MARL_FUSED(1, true); else MARL_FUSED(1, false); }
    else                 { if (q_all) MARL_FUSED(2, true); else MARL_FUSED(2, false); }
#undef MARL_FUSED
    return hipGetLastError();
}

}  // namespace

bool unroll_fused_fits(const NetFrags &net)
{
    if (net.kc1 > kFusedMaxKc1) return false;
    if (net.H == 64 && net.planes == 2) return FusedShape<64, 2>::lds_bytes(net.kc1) <= (size_t)kLdsLimit;
    if (net.H == 64 && net.planes == 1) return FusedShape<64, 1>::lds_bytes(net.kc1) <= (size_t)kLdsLimit;
    if (net.H == 128 && net.planes == 1) return FusedShape<128, 1>::lds_bytes(net.kc1) <= (size_t)kLdsLimit;
    return false;      // H = 128 with fp32 weights: the LDS buffers alone exceed a compute unit's 160 KiB
}

hipError_t launch_unroll_fused(const NetFrags &online, const NetFrags &target, bool two_nets, int B, int T,
                               const float *obs, const uint8_t *avail, const int32_t *actions, const float *reward,
                               const uint8_t *terminated, const uint8_t *filled, float gamma, float *q_taken,
                               float *next_max, float *td_target, float *q_all, hipStream_t stream)
{
#define MARL_GO(HH, PP)                                                                                             \
    return fused_dispatch<HH, PP>(online, target, two_nets, B, T, obs, avail, actions, reward, terminated, filled,  \
                                  gamma, q_taken, next_max, td_target, q_all, stream)
    if (online.H == 64 && online.planes == 2) MARL_GO(64, 2);
    if (online.H == 64 && online.planes == 1) MARL_GO(64, 1);
    if (online.H == 128 && online.planes == 1) MARL_GO(128, 1);
#undef MARL_GO
    return hipErrorInvalidValue;
}

}  // namespace marl
