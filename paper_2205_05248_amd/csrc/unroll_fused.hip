// Fused unroll + TD kernel for gfx950: one workgroup walks the T+1 slots of one tile of 16
// (episode, agent) rows for one network.  Every weight matrix stays on chip for the whole
// episode and no intermediate is written to global memory; per slot a workgroup reads its 16
// observation rows and the TD inputs, and writes the TD outputs.
//
// Where the weights live (H = 128, bf16: 278 KB in total):
//   W_hh   registers of the compute waves (each owns 32 hidden units: 3 gates x 2 blocks x H/32 k-steps)
//   W1     registers of the fc1 waves (each owns H/16/NF feature blocks x ceil(D/32) k-steps)
//   W_ih   LDS, copied once at kernel start (A operands are read from LDS at 16 bytes per lane)
//   W2     registers of the epilogue wave
//
// The work of a slot is cut into pipeline stages that run concurrently on different wavefronts,
// each on a different slot, and meet at ONE LDS-only barrier per slot.  In the step in which the
// recurrence handles slot s:
//
//   gates wave     first writes the observations of slot s+3 (loaded during the previous step) to
//                  LDS as bf16 operand fragments and issues the loads of slot s+4, then computes
//                  W_ih x + b for slot s+1 (x from LDS) and leaves the result in LDS in the
//                  accumulator form the recurrence reads;
//   fc1 waves      x = ReLU(W1 o + b1[agent]) for slot s+2, observation fragments from LDS, x to
//                  LDS as the next operand;
//   compute waves  slot s of the recurrence: W_hh h, gates, new hidden state to LDS as operand;
//   epilogue wave  fc2 / TD step of slot s-1.
//
// Only the recurrence is a dependent chain; the other stages are throughput work that hides
// under it.  Tiles of 16 rows (16x16x32 MFMAs) rather than 32 give twice as many workgroups, so
// that episode batches of a few thousand rows still occupy every compute unit, and halve the
// length of the chain per slot.
//
// Every LDS buffer is double-buffered on the parity of the slot it holds; a buffer written in
// step s was last read in step s-1 and is first read in step s+1.
#include <hip/hip_runtime.h>

#include "mfma16_tile.h"
#include "unroll_common.h"

namespace marl {

constexpr int kFusedLead = 4;         // steps before slot 0 enters the recurrence
constexpr int kLdsLimit = 160 * 1024;

template <int H, int P> struct Fused16 {
    static constexpr int FBK = H / 16;                 // feature blocks of the hidden layer
    static constexpr int KS = H / 32;                  // k-steps over the hidden layer
    static constexpr int NC = H / 32;                  // compute waves
    static constexpr int NF = H == 128 ? 2 : 1;        // fc1 waves
    static constexpr int NG = H == 128 ? 1 : 2;        // gates waves (the first one also moves the observations)
    static constexpr int kEpilogue = NC, kGates = NC + 1, kFc1 = NC + 1 + NG, kWaves = NC + 1 + NG + NF;
    static constexpr int NBF = FBK / NF;               // fc1 feature blocks per fc1 wave
    static constexpr int kKs1Max = 40 / (NBF * P);     // observation k-steps whose W1 fragments fit 160 registers
    static constexpr int kFrag = P * 1024;             // bytes of one fragment (all planes)
    static constexpr int kGiBlock = P == 1 ? 512 : 1024;   // one 16x16 gate-input block: bf16 / fp32 accumulator form
    static constexpr int kGiBytes = 3 * FBK * kGiBlock;
    // Gate blocks [0, kEpiBlocks) are computed by the epilogue wave, [kEpiBlocks, kGate1Blocks) by
    // the first gates wave and the rest by the second one, if there is one: the split evens out
    // the work of the wavefronts.
    static constexpr int kEpiBlocks = H == 128 ? 4 : 0;
    static constexpr int kGate1Blocks = H == 128 ? 3 * FBK : 4;
    // LDS layout (byte offsets)
    static constexpr int oWih = 0;                                  // [3 FBK][KS][P][64] bf16x8
    static constexpr int oGi = oWih + 3 * FBK * KS * kFrag;         // [2][3 FBK][kGiBlock]
    static constexpr int oH = oGi + 2 * kGiBytes;                   // [2][KS][P][64] bf16x8
    static constexpr int oX = oH + 2 * KS * kFrag;                  // [2][KS][P][64] bf16x8
    static constexpr int oGBias = oX + 2 * KS * kFrag;              // [3 H] floats: b_ir + b_hr, b_iz + b_hz, b_in
    static constexpr int oB2 = oGBias + 3 * H * 4;                  // [64] floats
    static constexpr int oObs = oB2 + 256;                          // [2][ks1][P][64] bf16x8
    static constexpr size_t lds_bytes(int ks1) { return (size_t)oObs + (size_t)2 * ks1 * kFrag; }
};

constexpr int fused_threads(int H) { return 64 * (H / 32 + 1 + (H == 128 ? 1 : 2) + (H == 128 ? 2 : 1)); }

// gate-input block <-> LDS
template <int P>
__device__ __forceinline__ void store_gi16(char *dst, int lane, const f32x4 &v)
{
    if constexpr (P == 1) {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        const bf16x4 t = {(__bf16)v[0], (__bf16)v[1], (__bf16)v[2], (__bf16)v[3]};
        *reinterpret_cast<bf16x4 *>(dst + lane * 8) = t;
    } else {
        *reinterpret_cast<f32x4 *>(dst + lane * 16) = v;
    }
}

template <int P>
__device__ __forceinline__ f32x4 load_gi16(const char *src, int lane)
{
    if constexpr (P == 1) {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        const bf16x4 t = *reinterpret_cast<const bf16x4 *>(src + lane * 8);
        const f32x4 v = {(float)t[0], (float)t[1], (float)t[2], (float)t[3]};
        return v;
    } else {
        return *reinterpret_cast<const f32x4 *>(src + lane * 16);
    }
}

// W_ih x + b for gate blocks [B0, B1) of one slot: x and the weight fragments come from LDS, the
// results go back to LDS for the compute waves.  Blocks are taken four at a time and k-step by
// k-step, so that an accumulator is touched by every fourth MFMA only (a dependent MFMA cannot
// issue before its predecessor has left the pipe).  The four fragments of a k-step are requested
// two k-steps ahead of their MFMAs; scheduling barriers keep the compiler from sinking those
// reads back next to their use.  A group's results are stored one k-step into the next group,
// when its last MFMAs have long finished; its accumulators start from the gate biases.
template <int H, int P, int B0, int B1>
__device__ __forceinline__ void gate_inputs(char *lds, int slot, int lane, int q4)
{
    using Sh = Fused16<H, P>;
    constexpr int KS = Sh::KS, GB = 4, NG = (B1 - B0) / GB, NT = NG * KS, DEPTH = 3;
    constexpr int NACC = KS >= 3 ? 2 : 3;            // accumulator sets in rotation (see the bias request below)
    static_assert((B1 - B0) % GB == 0, "groups of four blocks");
    if constexpr (NG > 0) {
        const int buf = slot & 1;
        // The per-lane offsets are made opaque once per call: otherwise the compiler precomputes
        // one address register per fragment, keeps them across the slot loop and spills them.
        // Two bases because an LDS access encodes at most 64 KB of constant offset.
        uint32_t lane_off = lane * 16, lane_off_hi = lane * 16 + 65536;
        asm volatile("" : "+v"(lane_off), "+v"(lane_off_hi));
        const char *wih_lane = lds + Sh::oWih + lane_off, *wih_lane_hi = lds + Sh::oWih + lane_off_hi;
        const float *gb = reinterpret_cast<const float *>(lds + Sh::oGBias);
        char *gi_dst = lds + Sh::oGi + buf * Sh::kGiBytes;
        Frag<P> x[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const bf16x8 *src = reinterpret_cast<const bf16x8 *>(lds + Sh::oX) + (size_t)((buf * KS + ks) * P) * 64 + lane;
            x[ks].hi = src[0];
            if constexpr (P == 2) x[ks].lo = src[64];
        }
        WFrag<P> w[DEPTH][GB];
        f32x4 acc[NACC][GB];
        auto request = [&](int t) {                  // fragments of step t = (group, k-step); a group's biases with its first step
            const int g = t / KS, ks = t % KS;
#pragma unroll
            for (int j = 0; j < GB; ++j) {
                const int blk = B0 + g * GB + j, off = (blk * KS + ks) * Sh::kFrag;
                w[t % DEPTH][j] = load_wfrag<P>(reinterpret_cast<const bf16x8 *>(off + Sh::kFrag <= 65536 ? wih_lane + off : wih_lane_hi + (off - 65536)));
                if (ks == 0) acc[g % NACC][j] = load_feature4(gb, blk, q4);
            }
        };
        auto store_group = [&](int g) {
#pragma unroll
            for (int j = 0; j < GB; ++j) store_gi16<P>(gi_dst + (B0 + g * GB + j) * Sh::kGiBlock, lane, acc[g % NACC][j]);
        };
#pragma unroll
        for (int t = 0; t < DEPTH - 1; ++t)
            if (t < NT) request(t);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            const int g = t / KS, ks = t % KS;
            if (t + DEPTH - 1 < NT) request(t + DEPTH - 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < GB; ++j) mma16<P>(acc[g % NACC][j], w[t % DEPTH][j], x[ks]);
            if (ks == 1 % KS && g > 0) store_group(g - 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        store_group(NG - 1);
    }
}

template <int H, int P, int AB, bool QALL>
__global__ __launch_bounds__(fused_threads(H), 2) void unroll_fused_kernel(
    NetFrags online, NetFrags target, int two_nets, int B, int T, const float *__restrict__ obs,
    const uint8_t *__restrict__ avail, const int32_t *__restrict__ actions, const float *__restrict__ reward,
    const uint8_t *__restrict__ terminated, const uint8_t *__restrict__ filled, float gamma,
    float *__restrict__ q_taken, float *__restrict__ next_max, float *__restrict__ td_target, float *__restrict__ q_all)
{
    using Sh = Fused16<H, P>;
    constexpr int FBK = Sh::FBK, KS = Sh::KS, LEAD = kFusedLead;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    typedef bf16x8 (*FragBuf)[KS][P][64];
    const FragBuf h_lds = reinterpret_cast<FragBuf>(lds + Sh::oH);
    const FragBuf x_lds = reinterpret_cast<FragBuf>(lds + Sh::oX);
    bf16x8 *const obuf = reinterpret_cast<bf16x8 *>(lds + Sh::oObs);        // [((slot & 1) ks1 + ks) P + p][64]
    bf16x8 *const wih_lds = reinterpret_cast<bf16x8 *>(lds + Sh::oWih);     // [((blk KS + ks) P + p)][64]

    const bool is_target = blockIdx.y == 1;
    const NetFrags &net = is_target ? target : online;
    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rt = blockIdx.x;
    const int N = net.N, D = net.D, A = net.A, S = T + 1;
    const int ks1 = (D + 31) / 32;
    const int rows = B * N;
    const int row = rt * 16 + c;
    const bool valid = row < rows;                     // rows past the end compute on row 0's inputs; results dropped
    const int b = valid ? row / N : 0, n = valid ? row % N : 0;

    // W_ih -> LDS, all waves.  Its first reader starts after at least three barriers.
    {
        constexpr int kVecs = 3 * FBK * KS * P * 64;
        for (int i = threadIdx.x; i < kVecs; i += fused_threads(H)) wih_lds[i] = net.wih_16[i];
    }
    // Steps run s = -LEAD .. T+1, one barrier at the end of each: LEAD + T + 2 barriers per wave.

    if (wave < Sh::NC) {
        // ---------------------------------------------------------------- compute wave
        // hidden units 32 w .. 32 w + 31 = feature blocks 2 w, 2 w + 1 = k-step w of the next operand
        const int w = wave;
        WFrag<P> whh[3][2][KS];
#pragma unroll
        for (int gate = 0; gate < 3; ++gate)
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    whh[gate][j][ks] = load_wfrag<P>(net.whh_16 + ((size_t)((gate * FBK + 2 * w + j) * KS + ks) * P) * 64 + lane);
        f32x4 bias_hn[2], hv[2];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            bias_hn[j] = load_feature4(net.bias_hn, 2 * w + j, q4);
#pragma unroll
            for (int r = 0; r < 4; ++r) hv[j][r] = 0.0f;
        }
        {
            const Frag<P> z0 = frag_of_pair<P>(hv[0], hv[1]);
            h_lds[0][w][0][lane] = z0.hi;
            if constexpr (P == 2) h_lds[0][w][1][lane] = z0.lo;
        }
        for (int i = 0; i < LEAD; ++i) lds_barrier();
        for (int it = 0; it <= T + 1; ++it) {
            if (it <= T) {
                const int cur = it & 1;
                const char *gi_cur = lds + Sh::oGi + cur * Sh::kGiBytes;
                f32x4 acc[3][2];
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    acc[0][j] = load_gi16<P>(gi_cur + (0 * FBK + 2 * w + j) * Sh::kGiBlock, lane);
                    acc[1][j] = load_gi16<P>(gi_cur + (1 * FBK + 2 * w + j) * Sh::kGiBlock, lane);
                    acc[2][j] = bias_hn[j];
                }
                Frag<P> hb[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    hb[ks].hi = h_lds[cur][ks][0][lane];
                    if constexpr (P == 2) hb[ks].lo = h_lds[cur][ks][1][lane];
                }
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
                        for (int j = 0; j < 2; ++j) mma16<P>(acc[gate][j], whh[gate][j][ks], hb[ks]);
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    const f32x4 ain = load_gi16<P>(gi_cur + (2 * FBK + 2 * w + j) * Sh::kGiBlock, lane);
                    hv[j] = gru_blend4(acc[0][j], acc[1][j], ain, acc[2][j], hv[j]);
                }
                const Frag<P> f = frag_of_pair<P>(hv[0], hv[1]);
                h_lds[cur ^ 1][w][0][lane] = f.hi;
                if constexpr (P == 2) h_lds[cur ^ 1][w][1][lane] = f.lo;
            }
            lds_barrier();
        }
    } else if (wave == Sh::kEpilogue) {
        // ---------------------------------------------------------------- epilogue wave
        const bool emit_online = !is_target, emit_target = is_target || !two_nets;
        float *const b2_lds = reinterpret_cast<float *>(lds + Sh::oB2);
        WFrag<P> w2[AB][KS];
#pragma unroll
        for (int ab = 0; ab < AB; ++ab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) w2[ab][ks] = load_wfrag<P>(net.w2_16 + ((size_t)(ab * KS + ks) * P) * 64 + lane);
        if (lane < 16 * AB) b2_lds[lane] = lane < A ? net.b2[lane] : 0.0f;
        // 32-bit element offsets (the host bounds every array to 2^30 elements)
        const uint32_t btn0 = (uint32_t)(b * T) * N + n;          // actions / outputs: + t N
        const uint32_t av0 = ((uint32_t)(b * S) * N + n) * A;     // avail / q_all:     + t N A
        const uint32_t bt0 = (uint32_t)(b * T);                   // per-episode flags: + t
        struct SlotIn { int u; uint32_t avail_raw[AB]; float reward; uint8_t on_filled, terminated, tg_filled; };
        auto fetch_slot = [&](int t) {          // inputs of slot t, requested one step before they are used
            SlotIn in{};
            if (t > T) return in;
            if (emit_online && t < T) {
                in.u = valid ? actions[btn0 + (uint32_t)t * N] : 0;
                in.on_filled = valid ? filled[bt0 + t] : 0;
            }
            if (emit_target && t >= 1) {
                if (A >= 4) issue_avail_loads16<AB>(avail + (valid ? av0 + (uint32_t)t * N * A : 0u), A, q4, in.avail_raw);
                in.reward = valid ? reward[bt0 + t - 1] : 0.0f;
                in.terminated = valid ? terminated[bt0 + t - 1] : 0;
                in.tg_filled = valid ? filled[bt0 + t - 1] : 0;
            }
            return in;
        };
        SlotIn nxt = fetch_slot(0);
        // lead-in steps: the epilogue wave's share of the gate inputs of slot 0 belongs to step -1
        for (int i = 0; i < LEAD; ++i) {
            if (i == LEAD - 1) gate_inputs<H, P, 0, Sh::kEpiBlocks>(lds, 0, lane, q4);
            lds_barrier();
        }
        for (int it = 0; it <= T + 1; ++it) {
            if (it + 1 <= T) gate_inputs<H, P, 0, Sh::kEpiBlocks>(lds, it + 1, lane, q4);
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
                        if (valid) store_q_row16<AB>(q_all + (av0 + (uint32_t)t * N * A), qv, A, q4);
                    }
                    if (t < T) {
                        const int u = min(max(in.u, 0), A - 1);
                        const float qu = pick_action_value16<AB>(qv, u, q4);
                        if (valid && q4 == 0) q_taken[btn0 + (uint32_t)t * N] = in.on_filled ? qu : 0.0f;
                    }
                }
                if (emit_target && t >= 1) {
                    const uint32_t slots =
                        A >= 4 ? avail_mask16<AB>(in.avail_raw, A, q4, valid)
                               : avail_mask_small16(avail + (valid ? av0 + (uint32_t)t * N * A : 0u), A, q4, valid);
                    const float best_q = masked_max16<AB>(qv, slots);
                    if (valid && q4 == 0) {
                        const uint32_t o = btn0 + (uint32_t)(t - 1) * N;
                        const float keep = in.terminated ? 0.0f : 1.0f;
                        const float y = in.reward + gamma * keep * best_q;
                        next_max[o] = in.tg_filled ? best_q : 0.0f;
                        td_target[o] = in.tg_filled ? y : 0.0f;
                    }
                }
            }
            lds_barrier();
        }
    } else if (wave == Sh::kGates) {
        // ---------------------------------------------------------------- gates wave (and observation loader)
        float *const gb = reinterpret_cast<float *>(lds + Sh::oGBias);       // private to this wave
        for (int i = lane; i < 3 * H; i += 64) {
            const int gate = i / H, j = i % H;       // = feature 16 (gate FBK + j / 16) + j % 16 of the stacked gates
            const float *src = gate == 0 ? net.bias_r : gate == 1 ? net.bias_z : net.bias_in;
            gb[i] = src[j];
        }
        // Observations: this lane's row, floats 32 ks + 8 q + 0..7 of k-step ks (the B operand's
        // k order).  Every k-step but the last lies wholly inside the row and is fetched as two
        // 16-byte loads at constant offsets from one address (only 4-byte alignment is assumed).
        // The last k-step, which may be partial, is fetched element by element from positions
        // clamped into the row; the weights are zero where the clamp changes a position.
        constexpr int KM = Sh::kKs1Max;
        const float *base = obs + ((size_t)b * S * N + n) * D + 8 * q4;      // slot 0
        const size_t slot_stride = (size_t)N * D;
        const int nfull = ks1 - 1;                   // k-steps handled by the vector path
        int last_off[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) last_off[i] = min(32 * nfull + 8 * q4 + i, D - 1) - 8 * q4;
        float stage[KM - 1 > 0 ? KM - 1 : 1][8], last[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) last[i] = 0.0f;

        for (int s = -LEAD; s <= T + 1; ++s) {
            const int ws = s + 3, ls = s + 4, gs = s + 1;
            if (ws >= 0 && ws <= T) {                // observations of slot ws: registers -> LDS
                bf16x8 *dst = obuf + (size_t)((ws & 1) * ks1) * P * 64 + lane;
                auto put = [&](bf16x8 *at, const float (&v)[8]) {
                    const Frag<P> f = to_frag<P>(v);
                    at[0] = f.hi;
                    if constexpr (P == 2) at[64] = f.lo;
                };
#pragma unroll
                for (int k = 0; k < KM - 1; ++k)
                    if (k < nfull) put(dst + (k * P) * 64, stage[k]);
                put(dst + (nfull * P) * 64, last);
            }
            if (ls >= 0 && ls <= T) {                // observations of slot ls: issue the loads
                const float *r = base + (size_t)ls * slot_stride;
#pragma unroll
                for (int k = 0; k < KM - 1; ++k)
                    if (k < nfull) {
                        f32x4 lo4, hi4;
                        __builtin_memcpy(&lo4, r + 32 * k, 16);
                        __builtin_memcpy(&hi4, r + 32 * k + 4, 16);
#pragma unroll
                        for (int i = 0; i < 4; ++i) { stage[k][i] = lo4[i]; stage[k][4 + i] = hi4[i]; }
                    }
#pragma unroll
                for (int i = 0; i < 8; ++i) last[i] = r[last_off[i]];
            }
            if (gs >= 0 && gs <= T) gate_inputs<H, P, Sh::kEpiBlocks, Sh::kGate1Blocks>(lds, gs, lane, q4);      // W_ih x + b of slot gs
            lds_barrier();
        }
    } else if (wave < Sh::kFc1) {
        // ---------------------------------------------------------------- second gates wave
        for (int s = -LEAD; s <= T + 1; ++s) {
            const int gs = s + 1;
            if (gs >= 0 && gs <= T) gate_inputs<H, P, Sh::kGate1Blocks, 3 * FBK>(lds, gs, lane, q4);
            lds_barrier();
        }
    } else {
        // ---------------------------------------------------------------- fc1 wave
        constexpr int NBF = Sh::NBF, KM = Sh::kKs1Max;
        const int f = wave - Sh::kFc1;               // owns feature blocks f NBF .. f NBF + NBF - 1 = k-steps f NBF/2 ..
        WFrag<P> w1[NBF][KM];
#pragma unroll
        for (int j = 0; j < NBF; ++j)
#pragma unroll
            for (int ks = 0; ks < KM; ++ks)
                if (ks < ks1) w1[j][ks] = load_wfrag<P>(net.w1_16 + ((size_t)((f * NBF + j) * ks1 + ks) * P) * 64 + lane);
        f32x4 b1v[NBF];
#pragma unroll
        for (int j = 0; j < NBF; ++j) b1v[j] = load_feature4(net.bias1 + (size_t)n * H, f * NBF + j, q4);
        auto obs_frag = [&](int slot, int ks) {
            const bf16x8 *src = obuf + (size_t)(((slot & 1) * ks1 + ks) * P) * 64 + lane;
            Frag<P> fr;
            fr.hi = src[0];
            if constexpr (P == 2) fr.lo = src[64];
            return fr;
        };
        // The first fc1 wave also pulls the observations of a later slot into L2 (one 4-byte load
        // per 128 bytes of every row, values unused), kTouchAhead steps before the gates wave loads
        // them for real: a first touch from HBM takes longer than one step, an L2 hit does not.
        constexpr int kTouchAhead = 4, TL = (KM * 32 + 127) / 128;          // loads per lane: the lane's lines q, q + 4, ...
        const float *touch_row = obs + ((size_t)b * S * N + n) * D;
        int touch_off[TL];
#pragma unroll
        for (int j = 0; j < TL; ++j) touch_off[j] = min(32 * (4 * j + q4), D - 1);
        uint32_t touched[kTouchAhead][TL] = {};
        // Register set c: what it fetched kTouchAhead steps ago must have arrived (the empty asm
        // consumes it) before it is loaded again.  The sets never move and the loop below is
        // unrolled over them, so no wait covers a load younger than kTouchAhead - 1 steps.
        auto touch = [&](uint32_t (&set)[TL], int s) {
            const float *r = touch_row + (size_t)min(max(s + 4 + kTouchAhead, 0), T) * N * D;   // ends: touched twice
#pragma unroll
            for (int j = 0; j < TL; ++j) asm volatile("" ::"v"(set[j]));
#pragma unroll
            for (int j = 0; j < TL; ++j) set[j] = __builtin_bit_cast(uint32_t, r[touch_off[j]]);
        };
        auto fc1_step = [&](int s) {
            const int slot = s + 2;
            if (slot >= 0 && slot <= T) {
                f32x4 acc[NBF];
#pragma unroll
                for (int j = 0; j < NBF; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[j][r] = 0.0f;
                // observation fragments are read two k-steps ahead of their MFMAs (LDS latency)
                Frag<P> bq[3];
                bq[0] = obs_frag(slot, 0);
                bq[1] = obs_frag(slot, min(1, ks1 - 1));
#pragma unroll
                for (int ks = 0; ks < KM; ++ks)
                    if (ks < ks1) {
                        bq[(ks + 2) % 3] = obs_frag(slot, min(ks + 2, ks1 - 1));
#pragma unroll
                        for (int j = 0; j < NBF; ++j) mma16<P>(acc[j], w1[j][ks], bq[ks % 3]);
                    }
#pragma unroll
                for (int j = 0; j < NBF; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[j][r] = fmaxf(acc[j][r] + b1v[j][r], 0.0f);
#pragma unroll
                for (int jj = 0; jj < NBF / 2; ++jj) {
                    const Frag<P> fr = frag_of_pair<P>(acc[2 * jj], acc[2 * jj + 1]);
                    x_lds[slot & 1][f * (NBF / 2) + jj][0][lane] = fr.hi;
                    if constexpr (P == 2) x_lds[slot & 1][f * (NBF / 2) + jj][1][lane] = fr.lo;
                }
            }
            lds_barrier();
        };
        int s = -LEAD;
        if (f == 0) {
            static_assert(kTouchAhead == 4, "the loop is unrolled over the register sets");
            for (; s + 3 <= T + 1; s += 4) {
                touch(touched[0], s);     fc1_step(s);
                touch(touched[1], s + 1); fc1_step(s + 1);
                touch(touched[2], s + 2); fc1_step(s + 2);
                touch(touched[3], s + 3); fc1_step(s + 3);
            }
        }
        for (; s <= T + 1; ++s) fc1_step(s);
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
    using Sh = Fused16<H, P>;
    const int tiles = (B * online.N + 15) / 16;
    const dim3 grid((unsigned)tiles, two_nets ? 2u : 1u), block(fused_threads(H));
    const size_t lds = Sh::lds_bytes((online.D + 31) / 32);
    const int two = two_nets ? 1 : 0;
    const int ab = (online.A + 15) / 16;
#define MARL_FUSED(ABLK, QA)                                                                                        \
    do {                                                                                                            \
        auto kernel = unroll_fused_kernel<H, P, ABLK, QA>;                                                          \
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),                               \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                 \
        if (err != hipSuccess) return err;                                                                          \
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, online, target, two, B, T, obs, avail, actions,        \
                           reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all);                 \
    } while (0)
#define MARL_FUSED_Q(ABLK) do { if (q_all) MARL_FUSED(ABLK, true); else MARL_FUSED(ABLK, false); } while (0)
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
