// The two wavefront roles that walk the T+1 slots of an episode tile (32 (episode, agent) rows)
// in both unroll kernels.  All wavefronts of the workgroup meet at one LDS-only barrier per
// slot; `lead` is the number of barriers the workgroup executes before slot 0 (pipeline fill of
// whoever produces the gate inputs).  After the lead, T + 2 more barriers follow.
//
//   compute_role   wave fb owns hidden units 32 fb .. 32 fb + 31: its slice of W_hh stays in
//                  registers for the whole episode; each slot it reads the full hidden state
//                  (operand form) and its gate inputs from LDS, does the hidden projection, the
//                  gates, and publishes its 32 new units.
//   epilogue_role  one slot behind: fc2 on the published hidden state (W2 in registers), then
//                  q_taken / masked max / TD target.
//
// LDS buffers (double-buffered across the barrier):
//   gi_lds   [2][3 H/32 blocks]  gate inputs of the slot in GiLayout<P> block form
//   h_lds    [2][H/16][P][64]    hidden state as B-operand fragments
#pragma once
#include "unroll_common.h"

namespace marl {

template <int H, int P>
__device__ __forceinline__ void compute_role(const NetFrags &net, int fb, int lane, int T, int lead, const char *gi_lds,
                                             bf16x8 (*h_lds)[H / 16][P][64])
{
    constexpr int FB = H / 32, KCH = H / 16;
    constexpr int kGiBytes = 3 * FB * GiLayout<P>::kBlockBytes;
    const int g = lane >> 5;
    bf16x8 w[3][KCH][P];
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc)
#pragma unroll
            for (int p = 0; p < P; ++p) w[gate][kc][p] = net.whh[((size_t)((gate * FB + fb) * KCH + kc) * P + p) * 64 + lane];
    const f32x16 bias_hn = load_feature_block(net.bias_hn, fb, g);
    f32x16 h;
#pragma unroll
    for (int r = 0; r < 16; ++r) h[r] = 0.0f;
    {
        const Frag<P> z0 = frag_of_half<P>(h, 0);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            h_lds[0][2 * fb + c][0][lane] = z0.hi;
            if constexpr (P == 2) h_lds[0][2 * fb + c][1][lane] = z0.lo;
        }
    }
    for (int i = 0; i < lead; ++i) lds_barrier();
    for (int it = 0; it <= T + 1; ++it) {
        if (it <= T) {
            const int cur = it & 1;
            const char *gi_cur = gi_lds + cur * kGiBytes;
            f32x16 acc[3];
#pragma unroll
            for (int gate = 0; gate < 2; ++gate)
                acc[gate] = load_gi_block<P>(gi_cur + (gate * FB + fb) * GiLayout<P>::kBlockBytes, lane);
            acc[2] = bias_hn;
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) {
                Frag<P> hb;
                hb.hi = h_lds[cur][kc][0][lane];
                if constexpr (P == 2) hb.lo = h_lds[cur][kc][1][lane];
#pragma unroll
                for (int gate = 0; gate < 3; ++gate) {
                    if constexpr (P == 2) {
                        acc[gate] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[gate][kc][1], hb.hi, acc[gate], 0, 0, 0);
                        acc[gate] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[gate][kc][0], hb.lo, acc[gate], 0, 0, 0);
                    }
                    acc[gate] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[gate][kc][0], hb.hi, acc[gate], 0, 0, 0);
                }
            }
            const f32x16 ain = load_gi_block<P>(gi_cur + (2 * FB + fb) * GiLayout<P>::kBlockBytes, lane);
            h = gru_blend(acc[0], acc[1], ain, acc[2], h);
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                const Frag<P> f = frag_of_half<P>(h, c);
                h_lds[cur ^ 1][2 * fb + c][0][lane] = f.hi;
                if constexpr (P == 2) h_lds[cur ^ 1][2 * fb + c][1][lane] = f.lo;
            }
        }
        lds_barrier();
    }
}

// Arrays of the TD step as the epilogue sees them.
struct TdArrays {
    const int32_t *episode_index;   // null: the input arrays hold the batch; else batch position b reads episode episode_index[b]
    int pool_episodes;              // episodes the input arrays hold (listed indices are clamped into it)
    const uint8_t *avail;
    const int32_t *actions;
    const float *reward;
    const uint8_t *terminated;
    const uint8_t *filled;
    float gamma;
    float *q_taken, *next_max, *td_target, *q_all;
    int mode;                       // TdMode
    int32_t *next_action;           // written under kTdSelect, read under kTdValue, unused otherwise
};

// emit_online: q_taken (and q_all); emit_target: next_max and td_target.  b2_lds: 32 MB2 floats
// owned by this wavefront.
template <int H, int P, int MB2, bool QALL>
__device__ __forceinline__ void epilogue_role(const NetFrags &net, const TdArrays &td, bool emit_online, bool emit_target,
                                              int rt, int lane, int B, int T, int lead, bf16x8 (*h_lds)[H / 16][P][64],
                                              float *b2_lds)
{
    constexpr int KCH = H / 16;
    const int g = lane >> 5, col = lane & 31;
    const int N = net.N, A = net.A, S = T + 1;
    const bool select = td.mode == kTdSelect, value = td.mode == kTdValue;
    emit_online = emit_online && !value;
    const int rows = B * N;
    const int row = rt * 32 + col;
    const bool valid = row < rows;
    const int b = valid ? row / N : 0, n = valid ? row % N : 0;
    bf16x8 w2[MB2][KCH][P];
#pragma unroll
    for (int mb = 0; mb < MB2; ++mb)
#pragma unroll
        for (int kc = 0; kc < KCH; ++kc)
#pragma unroll
            for (int p = 0; p < P; ++p) w2[mb][kc][p] = net.w2[((size_t)(mb * KCH + kc) * P + p) * 64 + lane];
    if (lane < 32 * MB2 / 2) {                 // the output bias lives in LDS, not in registers
        b2_lds[2 * lane] = net.b2[2 * lane];
        b2_lds[2 * lane + 1] = net.b2[2 * lane + 1];
    }

    // Per-slot inputs of the TD step, fetched one slot ahead so that their latency hides
    // behind the other waves' work.
    // 32-bit element offsets (the host bounds every array to 2^30 elements): uniform base
    // pointer + per-lane offset + per-slot stride.
    const int bi = td.episode_index ? min(max(td.episode_index[b], 0), td.pool_episodes - 1) : b;     // episode of the inputs
    const uint32_t btn0 = (uint32_t)(b * T) * N + n;          // outputs [B, T, N]:       + t N
    const uint32_t qa0 = ((uint32_t)(b * S) * N + n) * A;     // q_all [B, T+1, N, A]:    + t N A
    const uint32_t act0 = (uint32_t)(bi * T) * N + n;         // actions of the episode:  + t N
    const uint32_t av0 = ((uint32_t)(bi * S) * N + n) * A;    // avail of the episode:    + t N A
    const uint32_t bt0 = (uint32_t)(bi * T);                  // per-episode flags:       + t
    struct SlotIn { int u; uint32_t avail_raw[MB2 * 4]; float reward; uint8_t on_filled, terminated, tg_filled; };
    auto fetch_slot = [&](int t) {
        SlotIn in{};
        if (t > T) return in;
        if (emit_online && t < T) {
            in.u = valid ? td.actions[act0 + (uint32_t)t * N] : 0;
            in.on_filled = valid ? td.filled[bt0 + t] : 0;
        }
        if (emit_target && t >= 1) {
            if (value) in.u = valid ? td.next_action[btn0 + (uint32_t)(t - 1) * N] : -1;
            else if (A >= 4) issue_avail_loads<MB2>(td.avail + (valid ? av0 + (uint32_t)t * N * A : 0u), A, lane, in.avail_raw);
            in.reward = valid ? td.reward[bt0 + t - 1] : 0.0f;
            in.terminated = valid ? td.terminated[bt0 + t - 1] : 0;
            in.tg_filled = valid ? td.filled[bt0 + t - 1] : 0;
        }
        return in;
    };
    SlotIn nxt = fetch_slot(0);
    for (int i = 0; i < lead; ++i) lds_barrier();
    for (int it = 0; it <= T + 1; ++it) {
        if (it >= 1) {
            const int t = it - 1, cur = it & 1;          // h_t was published during iteration t
            const SlotIn in = nxt;
            nxt = fetch_slot(t + 1);
            f32x16 q[MB2];
#pragma unroll
            for (int mb = 0; mb < MB2; ++mb) q[mb] = load_feature_block(b2_lds, mb, g);
#pragma unroll
            for (int kc = 0; kc < KCH; ++kc) {
                Frag<P> hb;
                hb.hi = h_lds[cur][kc][0][lane];
                if constexpr (P == 2) hb.lo = h_lds[cur][kc][1][lane];
#pragma unroll
                for (int mb = 0; mb < MB2; ++mb) {
                    if constexpr (P == 2) {
                        q[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2[mb][kc][1], hb.hi, q[mb], 0, 0, 0);
                        q[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2[mb][kc][0], hb.lo, q[mb], 0, 0, 0);
                    }
                    q[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w2[mb][kc][0], hb.hi, q[mb], 0, 0, 0);
                }
            }
            if (emit_online) {
                if constexpr (QALL) {
                    if (valid) store_q_row<MB2>(td.q_all + (qa0 + (uint32_t)t * N * A), q, A, lane);
                }
                if (t < T) {
                    const int u = min(max(in.u, 0), A - 1);
                    const float qu = pick_action_value<MB2>(q, u, lane);
                    if (valid && g == 0) td.q_taken[btn0 + (uint32_t)t * N] = in.on_filled ? qu : 0.0f;
                }
            }
            if (emit_target && t >= 1) {
                const uint32_t o = btn0 + (uint32_t)(t - 1) * N;
                float best_q;
                if (value) {                       // the value of the action the other network chose
                    const float picked = pick_action_value<MB2>(q, min(max(in.u, 0), A - 1), lane);
                    best_q = in.u >= 0 ? picked : 0.0f;
                } else {
                    const uint32_t slots =
                        A >= 4 ? avail_mask_from_raw<MB2>(in.avail_raw, A, lane, valid)
                               : avail_mask_small(td.avail + (valid ? av0 + (uint32_t)t * N * A : 0u), A, lane, valid);
                    if (select) {
                        int best;
                        masked_argmax_slots<MB2>(q, slots, lane, best_q, best);
                        if (valid && g == 0) td.next_action[o] = best;
                    } else {
                        best_q = masked_max_slots<MB2>(q, slots);
                    }
                }
                if (!select && valid && g == 0) {
                    const float keep = in.terminated ? 0.0f : 1.0f;
                    const float y = in.reward + td.gamma * keep * best_q;
                    td.next_max[o] = in.tg_filled ? best_q : 0.0f;
                    td.td_target[o] = in.tg_filled ? y : 0.0f;
                }
            }
        }
        lds_barrier();
    }
}

}  // namespace marl
