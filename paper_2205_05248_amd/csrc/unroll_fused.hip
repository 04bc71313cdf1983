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

#include <type_traits>

#include "fused16_roles.h"

namespace marl {


// LDS of a launch: the shared layout, then the staging area of the epilogue's inputs, [2][4][64] words.
template <int H, int P> constexpr size_t unroll_lds_bytes(int ks1) { return Fused16<H, P>::lds_bytes(ks1) + 2 * 4 * 64 * 4; }

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

    // ---- the epilogue's per-slot inputs: the taken action, the flags, the reward and the availability bytes
    // kSelect / kValue: the two single-network launches of the double-estimator target
    constexpr bool kSelect = MODE == kTdSelect, kValue = MODE == kTdValue, kSave = MODE == kTdSave;
    // 32-bit element offsets (the host bounds every array to 2^30 elements)
    const uint32_t btn0 = (uint32_t)(b * T) * N + n;          // outputs [B, T, N]:       + t N
    const uint32_t qa0 = ((uint32_t)(b * S) * N + n) * A;     // q_all [B, T+1, N, A]:    + t N A
    const uint32_t act0 = (uint32_t)(bi * T) * N + n;         // actions of the episode:  + t N
    const uint32_t av0 = ((uint32_t)(bi * S) * N + n) * A;    // avail of the episode:    + t N A
    const uint32_t bt0 = (uint32_t)(bi * T);                  // per-episode flags:       + t
    // They are global loads whose latency is longer than a step, and the epilogue's own instruction stream cannot
    // hide it: its stores and loads are conditional, so any wait it needs covers everything in flight.  The loader
    // wave fetches them instead, beside the observations and a step earlier, the same number of loads every step
    // (positions clamped into the arrays, rows past the end read row 0), and hands them over in LDS:
    // epi[slot & 1][word][lane], words: 0 action, 1 flags (filled(t) | terminated(t-1) << 8 | filled(t-1) << 16),
    // 2 reward(t-1), 3 the lane's availability slots of slot t (avail_mask16, formed by the loader).
    // With two networks each workgroup's epilogue uses one half only - the online one the action and filled(t),
    // the target one the rest - and its loader fetches just that half (WANT_ONLINE / WANT_TARGET).
    struct SlotIn { int u; uint32_t flags; float reward; uint32_t slots; };
    struct SlotRaw { int u; uint32_t flags; float reward; uint32_t avail_raw[AB]; };
    constexpr int kEpiWords = 4;
    uint32_t *const epi = reinterpret_cast<uint32_t *>(lds + Sh::lds_bytes(ks1));
    auto fetch_slot = [&](int t, auto wide, auto want_online, auto want_target) {        // t in 0 .. T
        constexpr bool kOn = decltype(want_online)::value, kTg = decltype(want_target)::value;
        SlotRaw in{};
        if constexpr (!kSave) {
            const uint32_t tq = (uint32_t)min(t, T - 1), tp = (uint32_t)max(t - 1, 0);
            if constexpr (kValue) in.u = next_action[btn0 + tp * N];
            else if constexpr (kOn) in.u = actions[act0 + tq * N];
            if constexpr (kOn) in.flags = (uint32_t)filled[bt0 + tq];
            if constexpr (kTg) {
                in.flags |= (uint32_t)terminated[bt0 + tp] << 8 | (uint32_t)filled[bt0 + tp] << 16;
                in.reward = reward[bt0 + tp];
                if constexpr (decltype(wide)::value && !kValue)
                    issue_avail_loads16<AB>(avail + (av0 + (uint32_t)t * N * A), A, q4, in.avail_raw);
            }
        }
        return in;
    };
    auto stage_slot = [&](const SlotRaw &in, int t, auto wide, auto want_target) {
        uint32_t *at = epi + (size_t)(t & 1) * kEpiWords * 64 + lane;
        at[0] = (uint32_t)in.u;
        at[64] = in.flags;
        if constexpr (decltype(want_target)::value) {
            at[128] = __builtin_bit_cast(uint32_t, in.reward);
            if constexpr (decltype(wide)::value && !kValue && !kSave) at[192] = avail_mask16<AB>(in.avail_raw, A, q4, valid);
        }
    };
    auto staged_slot = [&](int t) {
        const uint32_t *at = epi + (size_t)(t & 1) * kEpiWords * 64 + lane;
        SlotIn in;
        in.u = (int)at[0];
        in.flags = at[64];
        in.reward = __builtin_bit_cast(float, at[128]);
        in.slots = at[192];
        return in;
    };

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
        gru.settle_weights();
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
        const bool emit_online = !is_target && !kValue && !kSave, emit_target = (is_target || !two_nets) && !kSave;
        float *const b2_lds = reinterpret_cast<float *>(lds + Sh::oB2);
        WFrag<P> w2[AB][KS];
#pragma unroll
        for (int ab = 0; ab < AB; ++ab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) w2[ab][ks] = load_wfrag<P>(net.w2_16 + ((size_t)(ab * KS + ks) * P) * 64 + lane);
        if (lane < 16 * AB) b2_lds[lane] = lane < A ? net.b2[lane] : 0.0f;
        // the weights have arrived before the loop starts: a wait for them inside it would also cover the loop's own loads
#pragma unroll
        for (int ab = 0; ab < AB; ++ab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) settle(w2[ab][ks]);
        for (int i = 0; i < LEAD; ++i) lds_barrier();
        for (int it = 0; it <= T + 1; ++it) {
            if (it >= 1) {
                const int t = it - 1, cur = it & 1;          // h_t was published during iteration t
                const SlotIn in = staged_slot(t);
                const bool on_filled = (in.flags & 0xFFu) != 0, terminated_prev = (in.flags >> 8 & 0xFFu) != 0, tg_filled = (in.flags >> 16 & 0xFFu) != 0;
                f32x4 qv[AB];
#pragma unroll
                for (int ab = 0; ab < AB; ++ab) qv[ab] = load_feature4(b2_lds, ab, q4);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    Frag<P> hb;
                    hb.hi = h_lds[cur][ks][0][lane];
                    if constexpr (P == 2) hb.lo = h_lds[cur][ks][1][lane];
                    {
                        f32x4 *accs[AB];
                        const WFrag<P> *wf[AB];
#pragma unroll
                        for (int ab = 0; ab < AB; ++ab) {
                            accs[ab] = &qv[ab];
                            wf[ab] = &w2[ab][ks];
                        }
                        mma16_across<P, AB>(accs, wf, hb);
                    }
                }
                if (emit_online) {
                    if constexpr (QALL) {
                        if (valid) store_q_row16<AB>(q_all + (qa0 + (uint32_t)t * N * A), qv, A, q4);
                    }
                    if (t < T) {
                        const int u = min(max(in.u, 0), A - 1);
                        const float qu = pick_action_value16<AB>(qv, u, q4);
                        if (valid && q4 == 0) q_taken[btn0 + (uint32_t)t * N] = on_filled ? qu : 0.0f;
                    }
                }
                if (emit_target && t >= 1) {
                    const uint32_t o = btn0 + (uint32_t)(t - 1) * N;
                    float best_q;
                    if constexpr (kValue) {               // the value of the action the other network chose
                        const float picked = pick_action_value16<AB>(qv, min(max(in.u, 0), A - 1), q4);
                        best_q = in.u >= 0 ? picked : 0.0f;      // -1: the other network found no action available
                    } else {
                        const uint32_t slots =
                            A >= 4 ? in.slots
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
                        const float keep = terminated_prev ? 0.0f : 1.0f;
                        const float y = in.reward + gamma * keep * best_q;
                        next_max[o] = tg_filled ? best_q : 0.0f;
                        td_target[o] = tg_filled ? y : 0.0f;
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
        // Two register sets in turn: a step first issues the loads of the slot it will write in the next step, into
        // the set that step will read, then converts the set loaded a step ago.  The loads have a whole step to arrive.
        ObsRegs<H, P> set_a, set_b;
        SlotRaw epi_a{}, epi_b{};                    // the epilogue's inputs of a slot, in turn like the observation sets
        auto loader_step = [&](const ObsRegs<H, P> &ready, ObsRegs<H, P> &refill, const SlotRaw &epi_ready, SlotRaw &epi_refill,
                               int s, auto wide, auto want_online, auto want_target) {
            const int ws = s + 2, ls = ws + 1;
            st.load(refill, base + (size_t)min(max(ls, 0), T) * slot_stride);       // every step the same number of loads (the ends load a slot again)
            epi_refill = fetch_slot(min(max(s + 1, 0), T), wide, want_online, want_target);     // slot s + 1: staged in the next step, read by the epilogue in step s + 2
            if (ws >= 0 && ws <= T) st.write(ready, obuf + (size_t)((ws & 1) * ks1) * P * 64 + lane);     // registers -> LDS
            if (s >= 0 && s <= T) stage_slot(epi_ready, s, wide, want_target);
            lds_barrier();
        };
        auto loader_loop = [&](auto wide, auto want_online, auto want_target) {
            int s = -LEAD;
            for (; s + 1 <= T + 1; s += 2) {
                loader_step(set_a, set_b, epi_a, epi_b, s, wide, want_online, want_target);
                loader_step(set_b, set_a, epi_b, epi_a, s + 1, wide, want_online, want_target);
            }
            if (s <= T + 1) loader_step(set_a, set_b, epi_a, epi_b, s, wide, want_online, want_target);
        };
        using Yes = std::true_type;
        using No = std::false_type;
        // which half the workgroup's epilogue uses (see emit_online / emit_target there)
        const bool need_online = !is_target && !kValue, need_target = is_target || !two_nets;
        if (A >= 4) {
            if (need_online && need_target) loader_loop(Yes{}, Yes{}, Yes{});
            else if (need_online) loader_loop(Yes{}, Yes{}, No{});
            else loader_loop(Yes{}, No{}, Yes{});
        } else {
            if (need_online && need_target) loader_loop(No{}, Yes{}, Yes{});
            else if (need_online) loader_loop(No{}, Yes{}, No{});
            else loader_loop(No{}, No{}, Yes{});
        }
    } else {
        // ---------------------------------------------------------------- fc1 wave
        const int f = wave - Sh::kFc1;
        Fc1Wave<H, P> fc1;
        fc1.load(net, f, ks1, lane);
        f32x4 b1v[Sh::NBF];
        Fc1Wave<H, P>::load_bias(net, f, n, q4, b1v);
        fc1.settle_weights(ks1);
#pragma unroll
        for (int j = 0; j < Sh::NBF; ++j) asm volatile("" ::"v"(b1v[j]));
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
    const size_t lds = unroll_lds_bytes<H, P>((online.D + 31) / 32);
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
    return ks1 <= Fused16<H, P>::kKs1Max && unroll_lds_bytes<H, P>(ks1) <= (size_t)kLdsLimit;
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
