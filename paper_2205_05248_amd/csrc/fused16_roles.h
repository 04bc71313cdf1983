// The per-wavefront building blocks the two fused kernels share (unroll_fused.hip walks the
// slots of an episode tile, act_fused.hip a run of tiles; per item the work is the same):
//
//   GruWave    a compute wave: its slice of W_hh in registers, W_ih fragments from LDS, both GRU
//              products, the gates, and the new hidden state as next operand
//   Fc1Wave    an fc1 wave: its feature blocks of W1 in registers, x = ReLU(W1 o + b1[agent])
//   ObsStage   the loader's observation registers (ObsRegs): global memory -> registers -> bf16
//              operand fragments in LDS
//   ObsTouch   the reads that pull a later item's rows into L2 ahead of the loader
#pragma once
#include "fused16.h"

namespace marl {

// Weights are loaded into registers once, before a loop that also has global memory traffic of
// its own.  Consuming them here places the wait for their arrival before the loop; otherwise it
// sits at their first use inside the loop, where it would also cover whatever the previous
// iteration left in flight.
template <int P> __device__ __forceinline__ void settle(const WFrag<P> &w)
{
    asm volatile("" ::"v"(w.hi));
    if constexpr (P == 2) asm volatile("" ::"v"(w.lo));
}

template <int H, int P> struct GruWave {
    using Sh = Fused16<H, P>;
    static constexpr int FBK = Sh::FBK, KS = Sh::KS, NBC = Sh::NBC;
    typedef bf16x8 (*FragBuf)[KS][P][64];
    WFrag<P> whh[3][NBC][KS];
    f32x4 bias_hn[NBC];

    // w = index of the compute wave: feature blocks NBC w .. NBC w + NBC - 1, all three gates
    __device__ __forceinline__ void load(const NetFrags &net, int w, int lane, int q4)
    {
#pragma unroll
        for (int gate = 0; gate < 3; ++gate)
#pragma unroll
            for (int j = 0; j < NBC; ++j)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    whh[gate][j][ks] = load_wfrag<P>(net.whh_16 + ((size_t)((gate * FBK + NBC * w + j) * KS + ks) * P) * 64 + lane);
#pragma unroll
        for (int j = 0; j < NBC; ++j) bias_hn[j] = load_feature4(net.bias_hn, NBC * w + j, q4);
    }

    __device__ __forceinline__ void settle_weights() const
    {
#pragma unroll
        for (int gate = 0; gate < 3; ++gate)
#pragma unroll
            for (int j = 0; j < NBC; ++j)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) settle(whh[gate][j][ks]);
#pragma unroll
        for (int j = 0; j < NBC; ++j) asm volatile("" ::"v"(bias_hn[j]));
    }

    // Gate biases (b_ir + b_hr, b_iz + b_hz, b_in) -> LDS, by one wave; read after a barrier.
    static __device__ __forceinline__ void stage_gate_biases(char *lds, const NetFrags &net, int lane)
    {
        float *const gb = reinterpret_cast<float *>(lds + Sh::oGBias);
        for (int i = lane; i < 3 * H; i += 64) {
            const int gate = i / H, j = i % H;       // = feature 16 (gate FBK + j / 16) + j % 16 of the stacked gates
            const float *src = gate == 0 ? net.bias_r : gate == 1 ? net.bias_z : net.bias_in;
            gb[i] = src[j];
        }
    }

    // One item: hv (this wave's units of the old state, fp32) -> the new state.  h_src / x_src:
    // the whole old state and the fc1 output as operand fragments in LDS.
    __device__ __forceinline__ void step(char *lds, int w, int lane, int q4, const bf16x8 (*h_src)[P][64],
                                         const bf16x8 (*x_src)[P][64], f32x4 (&hv)[NBC]) const
    {
        const float *gb = reinterpret_cast<const float *>(lds + Sh::oGBias);
        // W_ih fragments of this wave: two per-lane base addresses (an LDS access encodes at most
        // 64 KB of constant offset, the matrix may be larger) that already contain the wave's own
        // offset, so that every fragment is base + compile-time constant and costs no address
        // arithmetic.  The bases are made opaque once per item: otherwise the compiler precomputes
        // one address register per fragment and keeps them all across the loop.
        uint32_t lane_off = lane * 16 + (NBC * w * KS) * Sh::kFrag, lane_off_hi = lane_off + 65536;
        asm volatile("" : "+v"(lane_off), "+v"(lane_off_hi));
        const char *wih_lane = lds + Sh::oWih + lane_off, *wih_lane_hi = lds + Sh::oWih + lane_off_hi;
        WFrag<P> wi[2][3][NBC];              // W_ih fragments of two k-steps in rotation
        auto request = [&](int ks) {
#pragma unroll
            for (int gate = 0; gate < 3; ++gate)
#pragma unroll
                for (int j = 0; j < NBC; ++j) {
                    const int off = ((gate * FBK + j) * KS + ks) * Sh::kFrag;      // beyond the wave's own offset
                    wi[ks % 2][gate][j] = load_wfrag<P>(reinterpret_cast<const bf16x8 *>(
                        off + Sh::kFrag <= 65536 ? wih_lane + off : wih_lane_hi + (off - 65536)));
                }
        };
        Frag<P> hb[KS], x[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            hb[ks].hi = h_src[ks][0][lane];
            if constexpr (P == 2) hb[ks].lo = h_src[ks][1][lane];
        }
        f32x4 acc_r[NBC], acc_z[NBC], acc_in[NBC], acc_hn[NBC];
#pragma unroll
        for (int j = 0; j < NBC; ++j) {
            acc_r[j] = load_feature4(gb, 0 * FBK + NBC * w + j, q4);
            acc_z[j] = load_feature4(gb, 1 * FBK + NBC * w + j, q4);
            acc_in[j] = load_feature4(gb, 2 * FBK + NBC * w + j, q4);
            acc_hn[j] = bias_hn[j];
        }
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            x[ks].hi = x_src[ks][0][lane];
            if constexpr (P == 2) x[ks].lo = x_src[ks][1][lane];
        }
        request(0);
        request(1);
        __builtin_amdgcn_sched_barrier(0);
        // per k-step: the hidden product from registers, then the input product whose fragments
        // were requested two k-steps earlier; scheduling barriers keep the compiler from sinking
        // the requests back next to their use (LDS latency is several MFMAs long)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
            for (int j = 0; j < NBC; ++j) {
                f32x4 *const acc[3] = {&acc_r[j], &acc_z[j], &acc_hn[j]};
                const WFrag<P> *const wf[3] = {&whh[0][j][ks], &whh[1][j][ks], &whh[2][j][ks]};
                mma16_across<P, 3>(acc, wf, hb[ks]);
            }
#pragma unroll
            for (int j = 0; j < NBC; ++j) {
                f32x4 *const acc[3] = {&acc_r[j], &acc_z[j], &acc_in[j]};
                const WFrag<P> *const wf[3] = {&wi[ks % 2][0][j], &wi[ks % 2][1][j], &wi[ks % 2][2][j]};
                mma16_across<P, 3>(acc, wf, x[ks]);
            }
            __builtin_amdgcn_sched_barrier(0);
            if (ks + 2 < KS) request(ks + 2);
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int j = 0; j < NBC; ++j) hv[j] = gru_blend4(acc_r[j], acc_z[j], acc_in[j], acc_hn[j], hv[j]);
    }

    // The wave's units as next operand: two adjacent feature blocks make one k-step.  A wave with
    // two blocks writes a whole fragment, a wave with one block its half of every lane's 16 bytes.
    static __device__ __forceinline__ void publish(bf16x8 (*dst)[P][64], int w, int lane, const f32x4 (&hv)[NBC])
    {
        if constexpr (NBC == 2) {
            const Frag<P> f = frag_of_pair<P>(hv[0], hv[1]);
            dst[w][0][lane] = f.hi;
            if constexpr (P == 2) dst[w][1][lane] = f.lo;
        } else {
            typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
            bf16x4 hi, lo;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                hi[r] = (__bf16)hv[0][r];
                lo[r] = (__bf16)(hv[0][r] - (float)hi[r]);
            }
            char *at = reinterpret_cast<char *>(&dst[w / 2][0][lane]) + (w & 1) * 8;
            *reinterpret_cast<bf16x4 *>(at) = hi;
            if constexpr (P == 2) *reinterpret_cast<bf16x4 *>(at + 1024) = lo;
        }
    }
};

template <int H, int P> struct Fc1Wave {
    using Sh = Fused16<H, P>;
    static constexpr int NBF = Sh::NBF, KM = Sh::kKs1Max, KS = Sh::KS;
    WFrag<P> w1[NBF][KM];

    // f = index of the fc1 wave: feature blocks f NBF .. f NBF + NBF - 1 = k-steps f NBF/2 .. of x
    __device__ __forceinline__ void load(const NetFrags &net, int f, int ks1, int lane)
    {
#pragma unroll
        for (int j = 0; j < NBF; ++j)
#pragma unroll
            for (int ks = 0; ks < KM; ++ks)
                if (ks < ks1) w1[j][ks] = load_wfrag<P>(net.w1_16 + ((size_t)((f * NBF + j) * ks1 + ks) * P) * 64 + lane);
    }

    __device__ __forceinline__ void settle_weights(int ks1) const
    {
#pragma unroll
        for (int j = 0; j < NBF; ++j)
#pragma unroll
            for (int ks = 0; ks < KM; ++ks)
                if (ks < ks1) settle(w1[j][ks]);
    }

    static __device__ __forceinline__ void load_bias(const NetFrags &net, int f, int n, int q4, f32x4 (&b1v)[NBF])
    {
#pragma unroll
        for (int j = 0; j < NBF; ++j) b1v[j] = load_feature4(net.bias1 + (size_t)n * H, f * NBF + j, q4);
    }

    // One item: observation fragments obs_src[ks] (LDS) -> x fragments of this wave's blocks in x_dst.
    // SAVE: x also goes to elements 16 block + 0..3 of x_row (the caller has added the lane's 4 q; null: no store):
    // fp32 for a two-plane network, bf16 for a one-plane network (the rounding every reader of x applies anyway).
    template <bool SAVE = false>
    __device__ __forceinline__ void step(const bf16x8 *obs_src, int ks1, int f, int lane, const f32x4 (&b1v)[NBF],
                                         bf16x8 (*x_dst)[P][64], void *x_row = nullptr) const
    {
        auto obs_frag = [&](int ks) {
            const bf16x8 *src = obs_src + (size_t)(ks * P) * 64 + lane;
            Frag<P> fr;
            fr.hi = src[0];
            if constexpr (P == 2) fr.lo = src[64];
            return fr;
        };
        f32x4 acc[NBF];
#pragma unroll
        for (int j = 0; j < NBF; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[j][r] = 0.0f;
        // observation fragments are read two k-steps ahead of their MFMAs (LDS latency)
        Frag<P> bq[3];
        bq[0] = obs_frag(0);
        bq[1] = obs_frag(min(1, ks1 - 1));
#pragma unroll
        for (int ks = 0; ks < KM; ++ks)
            if (ks < ks1) {
                bq[(ks + 2) % 3] = obs_frag(min(ks + 2, ks1 - 1));
                {
                    f32x4 *accs[NBF];
                    const WFrag<P> *wf[NBF];
#pragma unroll
                    for (int j = 0; j < NBF; ++j) {
                        accs[j] = &acc[j];
                        wf[j] = &w1[j][ks];
                    }
                    mma16_across<P, NBF>(accs, wf, bq[ks % 3]);
                }
            }
#pragma unroll
        for (int j = 0; j < NBF; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[j][r] = fmaxf(acc[j][r] + b1v[j][r], 0.0f);
        if constexpr (SAVE) {
            if (x_row)
#pragma unroll
                for (int j = 0; j < NBF; ++j) {
                    if constexpr (P == 1) {
                        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                        bf16x4 v;
#pragma unroll
                        for (int r = 0; r < 4; ++r) v[r] = (__bf16)acc[j][r];
                        *reinterpret_cast<bf16x4 *>(static_cast<__bf16 *>(x_row) + 16 * (f * NBF + j)) = v;
                    } else {
                        *reinterpret_cast<f32x4 *>(static_cast<float *>(x_row) + 16 * (f * NBF + j)) = acc[j];
                    }
                }
        }
#pragma unroll
        for (int jj = 0; jj < NBF / 2; ++jj) {
            const Frag<P> fr = frag_of_pair<P>(acc[2 * jj], acc[2 * jj + 1]);
            x_dst[f * (NBF / 2) + jj][0][lane] = fr.hi;
            if constexpr (P == 2) x_dst[f * (NBF / 2) + jj][1][lane] = fr.lo;
        }
    }
};

// Observations of one item in the loader's registers.  A lane holds, per k-step, floats
// 32 ks + 8 q + 0..7 of its row (the B operand's k order).  Every k-step but the last lies wholly
// inside the row and is fetched as two 16-byte loads at constant offsets from one address (only
// 4-byte alignment is assumed).  The last k-step, which may be partial, is fetched element by
// element from positions clamped into the row; the weights are zero where the clamp changes a
// position.  ObsRegs is one item's worth of registers (a loader that runs several items ahead
// keeps several), ObsStage what all of them share.
template <int H, int P> struct ObsRegs {
    static constexpr int KM = Fused16<H, P>::kKs1Max;
    float stage[KM - 1 > 0 ? KM - 1 : 1][8], last[8];
};

template <int H, int P> struct ObsStage {
    static constexpr int KM = Fused16<H, P>::kKs1Max;
    int last_off[8];
    int nfull;                                       // k-steps handled by the vector path

    __device__ __forceinline__ void init(int D, int ks1, int q4)
    {
        nfull = ks1 - 1;
#pragma unroll
        for (int i = 0; i < 8; ++i) last_off[i] = min(32 * nfull + 8 * q4 + i, D - 1) - 8 * q4;
    }

    // row8 = the lane's row + 8 q
    __device__ __forceinline__ void load(ObsRegs<H, P> &r, const float *row8) const
    {
#pragma unroll
        for (int k = 0; k < KM - 1; ++k)
            if (k < nfull) {
                f32x4 lo4, hi4;
                __builtin_memcpy(&lo4, row8 + 32 * k, 16);
                __builtin_memcpy(&hi4, row8 + 32 * k + 4, 16);
#pragma unroll
                for (int i = 0; i < 4; ++i) { r.stage[k][i] = lo4[i]; r.stage[k][4 + i] = hi4[i]; }
            }
#pragma unroll
        for (int i = 0; i < 8; ++i) r.last[i] = row8[last_off[i]];
    }

    static __device__ __forceinline__ void put(bf16x8 *at, const float (&v)[8])
    {
        const Frag<P> f = to_frag<P>(v);
        at[0] = f.hi;
        if constexpr (P == 2) at[64] = f.lo;
    }

    // dst = this lane's slot in the item's first fragment
    __device__ __forceinline__ void write(const ObsRegs<H, P> &r, bf16x8 *dst) const
    {
#pragma unroll
        for (int k = 0; k < KM - 1; ++k)
            if (k < nfull) put(dst + (k * P) * 64, r.stage[k]);
        put(dst + (nfull * P) * 64, r.last);
    }
};

// Pulling rows into L2 ahead of the loader: one 4-byte load per 128 bytes of a row, values unused.
// A first touch from HBM takes longer than one pipeline step, an L2 hit does not.  EXTRA more
// values per set are for the caller's own touches.  Register set c: what it fetched kTouchAhead
// steps ago must have arrived (the empty asm consumes it) before it is loaded again; the sets
// never move and the caller's loop is unrolled over them, so no wait covers a younger load.
constexpr int kTouchAhead = 4;
template <int H, int P, int EXTRA> struct ObsTouch {
    static constexpr int TLO = (Fused16<H, P>::kKs1Max * 32 + 127) / 128, TL = TLO + EXTRA;
    int off[TLO];
    uint32_t set[kTouchAhead][TL] = {};

    __device__ __forceinline__ void init(int D, int q4)
    {
#pragma unroll
        for (int j = 0; j < TLO; ++j) off[j] = min(32 * (4 * j + q4), D - 1);      // the lane's lines q, q + 4, ...
    }

    __device__ __forceinline__ void consume(int c)
    {
#pragma unroll
        for (int j = 0; j < TL; ++j) asm volatile("" ::"v"(set[c][j]));
    }

    __device__ __forceinline__ void touch(int c, const float *row)
    {
#pragma unroll
        for (int j = 0; j < TLO; ++j) set[c][j] = __builtin_bit_cast(uint32_t, row[off[j]]);
    }
};

}  // namespace marl
