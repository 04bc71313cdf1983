// Fused unroll + TD kernel for gfx950: one workgroup walks the T+1 slots of one tile of 16
// (episode, agent) rows for one network.  Every weight matrix stays on chip for the whole
// episode and no intermediate is written to global memory; per slot a workgroup reads its 16
// observation rows and the TD inputs, and writes the TD outputs.
//
// Where the weights live (H = 128, bf16: 278 KB in total):
//   W_hh   registers of the compute waves (each owns H/64 feature blocks of 16 hidden units, all three gates)
//   W_ih   LDS, copied once at kernel start; each compute wave reads the fragments of its own
//          blocks from there every slot (A operands come from LDS at 16 bytes per lane)
//   W1     registers of the fc1 waves (each owns H/16/NF feature blocks x ceil(D/32) k-steps)
//   W2     registers of the epilogue wave
//
// The work of a slot is cut into pipeline stages that run concurrently on different wavefronts,
// each on a different slot, and meet at ONE LDS-only barrier per slot.  In the step in which the
// recurrence handles slot s:
//
//   loader wave    writes the observations of slot s+2 (loaded during the previous step) to LDS
//                  as bf16 operand fragments and issues the loads of slot s+3;
//   fc1 waves      x = ReLU(W1 o + b1[agent]) for slot s+1, observation fragments from LDS, x to
//                  LDS as the next operand; the first one also touches the observations of a
//                  later slot so that the loader's loads hit L2;
//   compute waves  slot s of the GRU: W_ih x + W_hh h + b for their hidden units, gates, new hidden
//                  state to LDS as operand;
//   epilogue wave  fc2 / TD step of slot s-1.
//
// Only the GRU is a dependent chain; the other stages are throughput work that hides under it.
// Tiles of 16 rows (16x16x32 MFMAs) rather than 32 give twice as many workgroups, so that
// episode batches of a few thousand rows still occupy every compute unit, and halve the length
// of the chain per slot.
//
// Every LDS buffer is double-buffered on the parity of the slot it holds; a buffer written in
// step s was last read in step s-1 and is first read in step s+1.
#include <hip/hip_runtime.h>

#include "fused16_roles.h"

namespace marl {

template <int H, int P, int AB, bool QALL, int MODE>
__global__ __launch_bounds__(fused_threads(H), 2) void unroll_fused_kernel(
    NetFrags online, NetFrags target, int two_nets, int B, int T, const int32_t *__restrict__ episode_index,
    int pool_episodes, const float *__restrict__ obs,
    const uint8_t *__restrict__ avail, const int32_t *__restrict__ actions, const float *__restrict__ reward,
    const uint8_t *__restrict__ terminated, const uint8_t *__restrict__ filled, float gamma,
    float *__restrict__ q_taken, float *__restrict__ next_max, float *__restrict__ td_target, float *__restrict__ q_all,
    int32_t *__restrict__ next_action, float *__restrict__ h_save, void *__restrict__ x_save)
{
    using Sh = Fused16<H, P>;
    constexpr int FBK = Sh::FBK, KS = Sh::KS, LEAD = kFusedLead;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    typedef bf16x8 (*FragBuf)[KS][P][64];
    const FragBuf h_lds = reinterpret_cast<FragBuf>(lds + Sh::oH);
    const FragBuf x_lds = reinterpret_cast<FragBuf>(lds + Sh::oX);
    bf16x8 *const obuf = reinterpret_cast<bf16x8 *>(lds + Sh::oObs);        // [((slot & 1) ks1 + ks) P + p][64]
    bf16x8 *const wih_lds = reinterpret_cast<bf16x8 *>(lds + Sh::oWih);     // [((blk KS + ks) P + p)][64]

    // Workgroup -> (tile, network).  With two networks the online and the target workgroup of a tile
    // sit eight apart in a block of sixteen consecutive workgroups: consecutive workgroups go round
    // the eight XCDs, so the pair shares one XCD's L2 (the second read of an observation line hits
    // there) and is dispatched at about the same time.
    const int rt = two_nets ? (int)(blockIdx.x >> 4) * 8 + (int)(blockIdx.x & 7) : (int)blockIdx.x;
    const bool is_target = two_nets && ((blockIdx.x >> 3) & 1);
    const int rows = B * online.N;
    if (rt * 16 >= rows) return;                          // padding of the last block of sixteen
    const NetFrags net = is_target ? target : online;     // by value: uniform, lives in scalar registers
    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int N = net.N, D = net.D, A = net.A, S = T + 1;
    const int ks1 = (D + 31) / 32;
    const int row = rt * 16 + c;
    const bool valid = row < rows;                     // rows past the end compute on row 0's inputs; results dropped
    const int b = valid ? row / N : 0, n = valid ? row % N : 0;         // position in the batch: outputs
    // episode of the input arrays: the batch position itself, or the listed episode of a larger pool
    const int bi = episode_index ? min(max(episode_index[b], 0), pool_episodes - 1) : b;

    // W_ih -> LDS, all waves.  Its first readers start after kFusedLead barriers.
    {
        constexpr int kVecs = 3 * FBK * KS * P * 64;
        for (int i = threadIdx.x; i < kVecs; i += fused_threads(H)) wih_lds[i] = net.wih_16[i];
    }
    // Steps run s = -LEAD .. T+1, one barrier at the end of each: LEAD + T + 2 barriers per wave.

    if (wave < Sh::NC) {
        // ---------------------------------------------------------------- compute wave
        const int w = wave;
        GruWave<H, P> gru;
        gru.load(net, w, lane, q4);
        if (w == 0) GruWave<H, P>::stage_gate_biases(lds, net, lane);
        f32x4 hv[Sh::NBC];                           // this wave's units of the hidden state, fp32
#pragma unroll
        for (int j = 0; j < Sh::NBC; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) hv[j][r] = 0.0f;
        GruWave<H, P>::publish(h_lds[0], w, lane, hv);
        // kTdSave / kTdKeep: this lane's units of its row's state, slot by slot (the online network's)
        constexpr bool kStores = MODE == kTdSave || MODE == kTdKeep;
        const bool stores = kStores && !is_target;
        float *h_row = nullptr;
        if constexpr (kStores) {
            h_row = h_save + ((size_t)b * S * N + n) * H + 16 * Sh::NBC * w + 4 * q4;
            if (valid && stores)
#pragma unroll
                for (int j = 0; j < Sh::NBC; ++j) *reinterpret_cast<f32x4 *>(h_row + 16 * j) = hv[j];
        }
        for (int i = 0; i < LEAD; ++i) lds_barrier();
        for (int it = 0; it <= T + 1; ++it) {
            if (it <= T) {
                const int cur = it & 1;
                gru.step(lds, w, lane, q4, h_lds[cur], x_lds[cur], hv);
                GruWave<H, P>::publish(h_lds[cur ^ 1], w, lane, hv);
                if constexpr (kStores) {
                    if (valid && stores && it < T)
#pragma unroll
                        for (int j = 0; j < Sh::NBC; ++j)
                            *reinterpret_cast<f32x4 *>(h_row + (size_t)(it + 1) * N * H + 16 * j) = hv[j];
                }
            }
            lds_barrier();
        }
    } else if (wave == Sh::kEpilogue) {
        // ---------------------------------------------------------------- epilogue wave
        // kSelect / kValue: the two single-network launches of the double-estimator target
        constexpr bool kSelect = MODE == kTdSelect, kValue = MODE == kTdValue, kSave = MODE == kTdSave;
        const bool emit_online = !is_target && !kValue && !kSave, emit_target = (is_target || !two_nets) && !kSave;
        float *const b2_lds = reinterpret_cast<float *>(lds + Sh::oB2);
        WFrag<P> w2[AB][KS];
#pragma unroll
        for (int ab = 0; ab < AB; ++ab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) w2[ab][ks] = load_wfrag<P>(net.w2_16 + ((size_t)(ab * KS + ks) * P) * 64 + lane);
        if (lane < 16 * AB) b2_lds[lane] = lane < A ? net.b2[lane] : 0.0f;
        // 32-bit element offsets (the host bounds every array to 2^30 elements)
        const uint32_t btn0 = (uint32_t)(b * T) * N + n;          // outputs [B, T, N]:       + t N
        const uint32_t qa0 = ((uint32_t)(b * S) * N + n) * A;     // q_all [B, T+1, N, A]:    + t N A
        const uint32_t act0 = (uint32_t)(bi * T) * N + n;         // actions of the episode:  + t N
        const uint32_t av0 = ((uint32_t)(bi * S) * N + n) * A;    // avail of the episode:    + t N A
        const uint32_t bt0 = (uint32_t)(bi * T);                  // per-episode flags:       + t
        struct SlotIn { int u; uint32_t avail_raw[AB]; float reward; uint8_t on_filled, terminated, tg_filled; };
        auto fetch_slot = [&](int t) {          // inputs of slot t, requested one step before they are used
            SlotIn in{};
            if (t > T) return in;
            if (emit_online && t < T) {
                in.u = valid ? actions[act0 + (uint32_t)t * N] : 0;
                in.on_filled = valid ? filled[bt0 + t] : 0;
            }
            if (emit_target && t >= 1) {
                if constexpr (kValue) in.u = valid ? next_action[btn0 + (uint32_t)(t - 1) * N] : -1;
                else if (A >= 4) issue_avail_loads16<AB>(avail + (valid ? av0 + (uint32_t)t * N * A : 0u), A, q4, in.avail_raw);
                in.reward = valid ? reward[bt0 + t - 1] : 0.0f;
                in.terminated = valid ? terminated[bt0 + t - 1] : 0;
                in.tg_filled = valid ? filled[bt0 + t - 1] : 0;
            }
            return in;
        };
        SlotIn nxt = fetch_slot(0);
        for (int i = 0; i < LEAD; ++i) lds_barrier();
        for (int it = 0; it <= T + 1; ++it) {
            if (it >= 1) {
                const int t = it - 1, cur = it & 1;          // h_t was published during iteration t
                const SlotIn in = nxt;
                nxt = fetch_slot(t + 1);
                f32x4 qv[AB];
#pragma unroll
                for (int ab = 0; ab < AB; ++ab) qv[ab] = load_feature4(b2_lds, ab, q4);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    Frag<P> hb;
                    hb.hi = h_lds[cur][ks][0][lane];
                    if constexpr (P == 2) hb.lo = h_lds[cur][ks][1][lane];
#pragma unroll
                    for (int ab = 0; ab < AB; ++ab) mma16<P>(qv[ab], w2[ab][ks], hb);
                }
                if (emit_online) {
                    if constexpr (QALL) {
                        if (valid) store_q_row16<AB>(q_all + (qa0 + (uint32_t)t * N * A), qv, A, q4);
                    }
                    if (t < T) {
                        const int u = min(max(in.u, 0), A - 1);
                        const float qu = pick_action_value16<AB>(qv, u, q4);
                        if (valid && q4 == 0) q_taken[btn0 + (uint32_t)t * N] = in.on_filled ? qu : 0.0f;
                    }
                }
                if (emit_target && t >= 1) {
                    const uint32_t o = btn0 + (uint32_t)(t - 1) * N;
                    float best_q;
                    if constexpr (kValue) {               // the value of the action the other network chose
                        const float picked = pick_action_value16<AB>(qv, min(max(in.u, 0), A - 1), q4);
                        best_q = in.u >= 0 ? picked : 0.0f;
                    } else {
                        const uint32_t slots =
                            A >= 4 ? avail_mask16<AB>(in.avail_raw, A, q4, valid)
                                   : avail_mask_small16(avail + (valid ? av0 + (uint32_t)t * N * A : 0u), A, q4, valid);
                        if constexpr (kSelect) {
                            int best;
                            masked_argmax16<AB, true>(qv, slots, q4, best_q, best);
                            if (valid && q4 == 0) next_action[o] = best;
                        } else {
                            best_q = masked_max16<AB>(qv, slots);
                        }
                    }
                    if (!kSelect && valid && q4 == 0) {
                        const float keep = in.terminated ? 0.0f : 1.0f;
                        const float y = in.reward + gamma * keep * best_q;
                        next_max[o] = in.tg_filled ? best_q : 0.0f;
                        td_target[o] = in.tg_filled ? y : 0.0f;
                    }
                }
            }
            lds_barrier();
        }
    } else if (wave == Sh::kLoader) {
        // ---------------------------------------------------------------- loader wave
        const float *base = obs + ((size_t)bi * S * N + n) * D + 8 * q4;     // the lane's row at slot 0
        const size_t slot_stride = (size_t)N * D;
        ObsStage<H, P> st;
        st.init(D, ks1, q4);
        ObsRegs<H, P> regs;
        for (int s = -LEAD; s <= T + 1; ++s) {
            const int ws = s + 2, ls = s + 3;
            if (ws >= 0 && ws <= T) st.write(regs, obuf + (size_t)((ws & 1) * ks1) * P * 64 + lane);     // registers -> LDS
            if (ls >= 0 && ls <= T) st.load(regs, base + (size_t)ls * slot_stride);                      // issue the loads
            lds_barrier();
        }
    } else {
        // ---------------------------------------------------------------- fc1 wave
        const int f = wave - Sh::kFc1;
        Fc1Wave<H, P> fc1;
        fc1.load(net, f, ks1, lane);
        f32x4 b1v[Sh::NBF];
        Fc1Wave<H, P>::load_bias(net, f, n, q4, b1v);
        const float *touch_row = obs + ((size_t)bi * S * N + n) * D;
        ObsTouch<H, P, 2> tch;
        tch.init(D, q4);
        auto touch = [&](int c, int s) {             // the slot the loader will load kTouchAhead steps from now
            const int slot = min(max(s + 3 + kTouchAhead, 0), T);                            // ends: touched twice
            tch.consume(c);
            tch.touch(c, touch_row + (size_t)slot * N * D);
            // and what the epilogues will read for that slot: the row's availability and action
            if constexpr (MODE != kTdSave) {
                tch.set[c][tch.TLO] = avail[(((size_t)bi * S + slot) * N + n) * A];
                tch.set[c][tch.TLO + 1] = (uint32_t)actions[((size_t)bi * T + min(slot, T - 1)) * N + n];
            }
        };
        auto fc1_step = [&](int s) {
            const int slot = s + 1;
            if (slot >= 0 && slot <= T) {
                if constexpr (MODE == kTdSave || MODE == kTdKeep)
                    fc1.template step<true>(obuf + (size_t)((slot & 1) * ks1) * P * 64, ks1, f, lane, b1v, x_lds[slot & 1],
                                            valid && !is_target ? static_cast<char *>(x_save) + ((((size_t)b * S + slot) * N + n) * H + 4 * q4) * (P == 1 ? 2 : 4)
                                                                : nullptr);
                else
                    fc1.step(obuf + (size_t)((slot & 1) * ks1) * P * 64, ks1, f, lane, b1v, x_lds[slot & 1]);
            }
            lds_barrier();
        };
        int s = -LEAD;
        // With two networks only the online workgroup touches: its partner on the tile reads the
        // same lines a few steps later and finds them in L2.  A partner that runs ahead misses,
        // waits for HBM and falls back behind, so the pair settles into that order by itself.
        if (f == 0 && !is_target) {
            static_assert(kTouchAhead == 4, "the loop is unrolled over the register sets");
            for (; s + 3 <= T + 1; s += 4) {
                touch(0, s);     fc1_step(s);
                touch(1, s + 1); fc1_step(s + 1);
                touch(2, s + 2); fc1_step(s + 2);
                touch(3, s + 3); fc1_step(s + 3);
            }
        }
        for (; s <= T + 1; ++s) fc1_step(s);
    }
}

// ------------------------------------------------------------------------------------------ host side
namespace {

template <int H, int P>
hipError_t fused_dispatch(const NetFrags &online, const NetFrags &target, bool two_nets, int B, int T,
                          const int32_t *episode_index, int pool_episodes, const float *obs, const uint8_t *avail, const int32_t *actions, const float *reward,
                          const uint8_t *terminated, const uint8_t *filled, float gamma, float *q_taken,
                          float *next_max, float *td_target, float *q_all, hipStream_t stream, TdMode mode,
                          int32_t *next_action, float *h_save, void *x_save)
{
    using Sh = Fused16<H, P>;
    const int tiles = (B * online.N + 15) / 16;
    const dim3 grid(two_nets ? (unsigned)((tiles + 7) / 8) * 16u : (unsigned)tiles), block(fused_threads(H));
    const size_t lds = Sh::lds_bytes((online.D + 31) / 32);
    const int two = two_nets ? 1 : 0;
    const int ab = (online.A + 15) / 16;
#define MARL_FUSED(ABLK, QA, MD)                                                                                    \
    do {                                                                                                            \
        auto kernel = unroll_fused_kernel<H, P, ABLK, QA, MD>;                                                      \
        hipError_t err = allow_large_lds<unroll_fused_kernel<H, P, ABLK, QA, MD>>(kLdsLimit);                       \
        if (err != hipSuccess) return err;                                                                          \
        launch_kernel(kernel, grid, block, lds, stream, online, target, two, B, T, episode_index, pool_episodes,      \
                           obs, avail, actions,                                                                      \
                           reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all, next_action,     \
                           h_save, x_save);                                                                         \
    } while (0)
#define MARL_FUSED_Q(ABLK)                                                                                          \
    do {                                                                                                            \
        if (mode == kTdSave) MARL_FUSED(ABLK, false, kTdSave);                                                      \
        else if (mode == kTdKeep) { if (q_all) MARL_FUSED(ABLK, true, kTdKeep); else MARL_FUSED(ABLK, false, kTdKeep); } \
        else if (mode == kTdValue) MARL_FUSED(ABLK, false, kTdValue);                                               \
        else if (mode == kTdSelect) { if (q_all) MARL_FUSED(ABLK, true, kTdSelect); else MARL_FUSED(ABLK, false, kTdSelect); } \
        else if (q_all) MARL_FUSED(ABLK, true, kTdPlain);                                                           \
        else MARL_FUSED(ABLK, false, kTdPlain);                                                                     \
    } while (0)
    switch (ab) {
    case 1: MARL_FUSED_Q(1); break;
    case 2: MARL_FUSED_Q(2); break;
    case 3: MARL_FUSED_Q(3); break;
    case 4: MARL_FUSED_Q(4); break;
    default: return hipErrorInvalidValue;
    }
#undef MARL_FUSED_Q
#undef MARL_FUSED
    return hipGetLastError();
}

template <int H, int P> bool fits(const NetFrags &net)
{
    const int ks1 = (net.D + 31) / 32;
    return ks1 <= Fused16<H, P>::kKs1Max && Fused16<H, P>::lds_bytes(ks1) <= (size_t)kLdsLimit;
}

}  // namespace

bool unroll_fused_fits(const NetFrags &net)
{
    if (net.A > 64) return false;
    if (net.H == 64 && net.planes == 2) return fits<64, 2>(net);
    if (net.H == 64 && net.planes == 1) return fits<64, 1>(net);
    if (net.H == 128 && net.planes == 1) return fits<128, 1>(net);
    return false;      // H = 128 with fp32 weights: W_ih alone exceeds a compute unit's LDS
}

hipError_t launch_unroll_fused(const NetFrags &online, const NetFrags &target, bool two_nets, int B, int T,
                               const int32_t *episode_index, int pool_episodes, const float *obs, const uint8_t *avail, const int32_t *actions, const float *reward,
                               const uint8_t *terminated, const uint8_t *filled, float gamma, float *q_taken,
                               float *next_max, float *td_target, float *q_all, hipStream_t stream, TdMode mode,
                               int32_t *next_action, float *h_save, void *x_save)
{
    if ((mode == kTdSelect || mode == kTdValue) && (two_nets || !next_action)) return hipErrorInvalidValue;
    if (mode == kTdSave && (two_nets || !h_save || !x_save)) return hipErrorInvalidValue;
    if (mode == kTdKeep && (!h_save || !x_save)) return hipErrorInvalidValue;
#define MARL_GO(HH, PP)                                                                                             \
    return fused_dispatch<HH, PP>(online, target, two_nets, B, T, episode_index, pool_episodes, obs, avail, actions, reward, terminated, filled,  \
                                  gamma, q_taken, next_max, td_target, q_all, stream, mode, next_action, h_save, x_save)
    if (online.H == 64 && online.planes == 2) MARL_GO(64, 2);
    if (online.H == 64 && online.planes == 1) MARL_GO(64, 1);
    if (online.H == 128 && online.planes == 1) MARL_GO(128, 1);
#undef MARL_GO
    return hipErrorInvalidValue;
}

}  // namespace marl
