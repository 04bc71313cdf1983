// Fused decision-step kernel for gfx950 on tiles of 16 (env, agent) rows.
//
// Same machine as the fused unroll (unroll_fused.hip): every weight stays on chip (W_hh, W1, W2 in
// registers, W_ih in LDS) and the work of a tile is a pipeline over wavefront roles that meet at
// one LDS-only barrier per step.  Here the pipeline runs over the workgroup's *tiles* instead of
// over the slots of an episode: a workgroup owns a run of consecutive tiles, and in the step in
// which the GRU handles item k (the k-th tile of the run)
//
//   loader wave    writes the observations of item k+2 and the incoming hidden state of item k+1
//                  (both loaded during the previous step) to LDS as bf16 operand fragments, and
//                  issues the loads of items k+3 / k+2;
//   fc1 waves      x = ReLU(W1 o + b1[agent]) for item k+1; the first one also touches the
//                  observations of a later item so that the loader's loads hit L2;
//   compute waves  item k of the GRU: W_ih x + W_hh h + b for their hidden units, gates, new hidden
//                  state to global memory (fp32) and to LDS (operand form);
//   epilogue wave  item k-1: fc2, Q store, availability mask, argmax, epsilon-greedy, action store.
//
// Nothing depends on the previous item, so the steps are pure throughput; the per-launch cost of
// loading the weights (once per workgroup) is amortised over the run of tiles.
#include <hip/hip_runtime.h>

#include "fused16.h"

namespace marl {

struct ActFusedArgs {
    NetFrags net;
    int rows;                   // E * N
    int tiles_per_group;        // consecutive tiles of 16 rows per workgroup
    const float *obs;
    const uint8_t *avail;
    const float *h_in;
    const uint8_t *reset;       // may be null
    const int32_t *step_t;
    float epsilon;
    uint64_t seed;
    float *h_out;
    int32_t *action;
    float *q_out;               // may be null
};

// Masked argmax of a row whose Q values are split over the four lanes c, c + 16, c + 32, c + 48;
// lowest index on ties; idx = -1 when nothing is available.
template <int AB>
__device__ __forceinline__ void masked_argmax16(const f32x4 (&qv)[AB], uint32_t slots, int q, float &best_q, int &best_idx)
{
    best_q = 0.0f; best_idx = -1;
#pragma unroll
    for (int ab = 0; ab < AB; ++ab)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const bool ok = (slots >> (4 * ab + r)) & 1u;
            if (ok && (best_idx < 0 || qv[ab][r] > best_q)) { best_q = qv[ab][r]; best_idx = 16 * ab + 4 * q + r; }
        }
#pragma unroll
    for (int m = 16; m <= 32; m <<= 1) {
        const float oq = __shfl_xor(best_q, m);
        const int oi = __shfl_xor(best_idx, m);
        if (oi >= 0 && (best_idx < 0 || oq > best_q || (oq == best_q && oi < best_idx))) { best_q = oq; best_idx = oi; }
    }
}

// Availability bits of the whole row (bit a = action a) from the four lanes' slot masks.
template <int AB>
__device__ __forceinline__ uint64_t row_avail_bits16(uint32_t slots, int q)
{
    uint64_t bits = 0;
#pragma unroll
    for (int ab = 0; ab < AB; ++ab) bits |= (uint64_t)((slots >> (4 * ab)) & 0xFu) << (16 * ab + 4 * q);
    uint32_t lo = (uint32_t)bits, hi = (uint32_t)(bits >> 32);
#pragma unroll
    for (int m = 16; m <= 32; m <<= 1) {
        lo |= __shfl_xor(lo, m);
        hi |= __shfl_xor(hi, m);
    }
    return ((uint64_t)hi << 32) | lo;
}

template <int H, int P, int AB>
__global__ __launch_bounds__(fused_threads(H), 2) void act_fused_kernel(const ActFusedArgs args)
{
    using Sh = Fused16<H, P>;
    constexpr int FBK = Sh::FBK, KS = Sh::KS, LEAD = kFusedLead;
    extern __shared__ __attribute__((aligned(16))) char lds[];
    typedef bf16x8 (*FragBuf)[KS][P][64];
    const NetFrags &net = args.net;
    const int N = net.N, D = net.D, A = net.A;
    const int ks1 = (D + 31) / 32;
    const FragBuf h_lds = reinterpret_cast<FragBuf>(lds + Sh::oH);                   // new hidden state, compute -> epilogue
    const FragBuf x_lds = reinterpret_cast<FragBuf>(lds + Sh::oX);
    const FragBuf hin_lds = reinterpret_cast<FragBuf>(lds + Sh::hin_offset(ks1));    // old hidden state, loader -> compute
    bf16x8 *const obuf = reinterpret_cast<bf16x8 *>(lds + Sh::oObs);
    bf16x8 *const wih_lds = reinterpret_cast<bf16x8 *>(lds + Sh::oWih);

    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rows = args.rows;
    const int tiles = (rows + 15) / 16;
    const int first = blockIdx.x * args.tiles_per_group;
    const int count = min(args.tiles_per_group, tiles - first);       // >= 1 by construction of the grid
    // item k (0 <= k < count) is tile first + k; items past the run re-use its last tile (reads only)
    auto item_row = [&](int k) { return (first + min(max(k, 0), count - 1)) * 16 + c; };
    // Steps run s = -LEAD .. count, one barrier at the end of each: LEAD + count + 1 barriers per wave.

    {
        constexpr int kVecs = 3 * FBK * KS * P * 64;
        for (int i = threadIdx.x; i < kVecs; i += fused_threads(H)) wih_lds[i] = net.wih_16[i];
    }

    if (wave < Sh::NC) {
        // ---------------------------------------------------------------- compute wave
        constexpr int NBC = Sh::NBC;
        const int w = wave;
        WFrag<P> whh[3][NBC][KS];
#pragma unroll
        for (int gate = 0; gate < 3; ++gate)
#pragma unroll
            for (int j = 0; j < NBC; ++j)
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    whh[gate][j][ks] = load_wfrag<P>(net.whh_16 + ((size_t)((gate * FBK + NBC * w + j) * KS + ks) * P) * 64 + lane);
        f32x4 bias_hn[NBC];
#pragma unroll
        for (int j = 0; j < NBC; ++j) bias_hn[j] = load_feature4(net.bias_hn, NBC * w + j, q4);
        float *const gb = reinterpret_cast<float *>(lds + Sh::oGBias);
        if (w == 0)
            for (int i = lane; i < 3 * H; i += 64) {
                const int gate = i / H, j = i % H;
                const float *src = gate == 0 ? net.bias_r : gate == 1 ? net.bias_z : net.bias_in;
                gb[i] = src[j];
            }
        for (int i = 0; i < LEAD; ++i) lds_barrier();
        for (int s = 0; s <= count; ++s) {
            if (s < count) {
                const int cur = s & 1;
                const int row = item_row(s);
                const bool valid = row < rows;
                const int rr = valid ? row : 0;
                const bool keep = !(args.reset && args.reset[rr / N]);
                // this wave's own units of the old state in fp32, for the blend
                f32x4 hv[NBC];
#pragma unroll
                for (int j = 0; j < NBC; ++j) {
                    const f32x4 t = *reinterpret_cast<const f32x4 *>(args.h_in + (size_t)rr * H + 16 * (NBC * w + j) + 4 * q4);
#pragma unroll
                    for (int r = 0; r < 4; ++r) hv[j][r] = keep ? t[r] : 0.0f;
                }
                uint32_t lane_off = lane * 16, lane_off_hi = lane * 16 + 65536;
                asm volatile("" : "+v"(lane_off), "+v"(lane_off_hi));
                const char *wih_lane = lds + Sh::oWih + lane_off, *wih_lane_hi = lds + Sh::oWih + lane_off_hi;
                WFrag<P> wi[2][3][NBC];
                auto request = [&](int ks) {
#pragma unroll
                    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
                        for (int j = 0; j < NBC; ++j) {
                            const int off = ((gate * FBK + NBC * w + j) * KS + ks) * Sh::kFrag;
                            wi[ks % 2][gate][j] = load_wfrag<P>(reinterpret_cast<const bf16x8 *>(
                                off + Sh::kFrag <= 65536 ? wih_lane + off : wih_lane_hi + (off - 65536)));
                        }
                };
                Frag<P> hb[KS], x[KS];
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    hb[ks].hi = hin_lds[cur][ks][0][lane];
                    if constexpr (P == 2) hb[ks].lo = hin_lds[cur][ks][1][lane];
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
                    x[ks].hi = x_lds[cur][ks][0][lane];
                    if constexpr (P == 2) x[ks].lo = x_lds[cur][ks][1][lane];
                }
                request(0);
                request(1);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                    for (int j = 0; j < NBC; ++j) {
                        mma16<P>(acc_r[j], whh[0][j][ks], hb[ks]);
                        mma16<P>(acc_z[j], whh[1][j][ks], hb[ks]);
                        mma16<P>(acc_hn[j], whh[2][j][ks], hb[ks]);
                    }
#pragma unroll
                    for (int j = 0; j < NBC; ++j) {
                        mma16<P>(acc_r[j], wi[ks % 2][0][j], x[ks]);
                        mma16<P>(acc_z[j], wi[ks % 2][1][j], x[ks]);
                        mma16<P>(acc_in[j], wi[ks % 2][2][j], x[ks]);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    if (ks + 2 < KS) request(ks + 2);
                    __builtin_amdgcn_sched_barrier(0);
                }
#pragma unroll
                for (int j = 0; j < NBC; ++j) {
                    hv[j] = gru_blend4(acc_r[j], acc_z[j], acc_in[j], acc_hn[j], hv[j]);
                    if (valid) *reinterpret_cast<f32x4 *>(args.h_out + (size_t)row * H + 16 * (NBC * w + j) + 4 * q4) = hv[j];
                }
                // the new state as operand for fc2 (two adjacent feature blocks make one k-step)
                if constexpr (NBC == 2) {
                    const Frag<P> f = frag_of_pair<P>(hv[0], hv[1]);
                    h_lds[cur][w][0][lane] = f.hi;
                    if constexpr (P == 2) h_lds[cur][w][1][lane] = f.lo;
                } else {
                    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                    bf16x4 hi, lo;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        hi[r] = (__bf16)hv[0][r];
                        lo[r] = (__bf16)(hv[0][r] - (float)hi[r]);
                    }
                    char *dst = reinterpret_cast<char *>(&h_lds[cur][w / 2][0][lane]) + (w & 1) * 8;
                    *reinterpret_cast<bf16x4 *>(dst) = hi;
                    if constexpr (P == 2) *reinterpret_cast<bf16x4 *>(dst + 1024) = lo;
                }
            }
            lds_barrier();
        }
    } else if (wave == Sh::kEpilogue) {
        // ---------------------------------------------------------------- epilogue wave
        float *const b2_lds = reinterpret_cast<float *>(lds + Sh::oB2);
        WFrag<P> w2[AB][KS];
#pragma unroll
        for (int ab = 0; ab < AB; ++ab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) w2[ab][ks] = load_wfrag<P>(net.w2_16 + ((size_t)(ab * KS + ks) * P) * 64 + lane);
        if (lane < 16 * AB) b2_lds[lane] = lane < A ? net.b2[lane] : 0.0f;
        struct ItemIn { uint32_t avail_raw[AB]; int step; };
        auto fetch_item = [&](int k) {          // inputs of item k, requested one step before they are used
            ItemIn in{};
            const int row = item_row(k);
            const int rr = row < rows ? row : 0;
            if (A >= 4) issue_avail_loads16<AB>(args.avail + (size_t)rr * A, A, q4, in.avail_raw);
            in.step = args.step_t[rr / N];
            return in;
        };
        ItemIn nxt = fetch_item(0);
        for (int i = 0; i < LEAD; ++i) lds_barrier();
        for (int s = 0; s <= count; ++s) {
            if (s >= 1) {
                const int k = s - 1, cur = k & 1;
                const ItemIn in = nxt;
                nxt = fetch_item(k + 1);
                const int row = item_row(k);
                const bool valid = row < rows;
                const int rr = valid ? row : 0;
                const int e = rr / N, n = rr % N;
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
                if (args.q_out && valid) store_q_row16<AB>(args.q_out + (size_t)row * A, qv, A, q4);
                const uint32_t slots = A >= 4 ? avail_mask16<AB>(in.avail_raw, A, q4, valid)
                                              : avail_mask_small16(args.avail + (size_t)rr * A, A, q4, valid);
                float best_q; int best;
                masked_argmax16<AB>(qv, slots, q4, best_q, best);
                const uint64_t bits = row_avail_bits16<AB>(slots, q4);
                if (valid && q4 == 0) {
                    if (best < 0) best = 0;
                    args.action[row] = eps_greedy_pick(best, bits, args.epsilon, args.seed, (uint32_t)e, (uint32_t)n, (uint32_t)in.step);
                }
            }
            lds_barrier();
        }
    } else if (wave == Sh::kLoader) {
        // ---------------------------------------------------------------- loader wave
        // Observations: this lane's row, floats 32 ks + 8 q + 0..7 of k-step ks (the B operand's
        // k order).  Every k-step but the last lies wholly inside the row and is fetched as two
        // 16-byte loads (only 4-byte alignment is assumed).  The last k-step, which may be partial,
        // is fetched element by element from positions clamped into the row; the weights are
        // zero where the clamp changes a position.
        // Hidden state: the operand of k-step ks wants features 32 ks + 16 (idx / 4) + 4 q + idx % 4,
        // i.e. two aligned groups of four floats.
        constexpr int KM = Sh::kKs1Max;
        const int nfull = ks1 - 1;
        int last_off[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) last_off[i] = min(32 * nfull + 8 * q4 + i, D - 1) - 8 * q4;
        float stage[KM - 1 > 0 ? KM - 1 : 1][8], last[8], hstage[KS][8];
#pragma unroll
        for (int i = 0; i < 8; ++i) last[i] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int i = 0; i < 8; ++i) hstage[ks][i] = 0.0f;
        auto put = [&](bf16x8 *at, const float (&v)[8]) {
            const Frag<P> f = to_frag<P>(v);
            at[0] = f.hi;
            if constexpr (P == 2) at[64] = f.lo;
        };
        for (int s = -LEAD; s <= count; ++s) {
            const int ws = s + 2, ls = s + 3;        // observations: item written / loaded in this step
            const int hw = s + 1, hl = s + 2;        // hidden state: one item closer to its use
            if (ws >= 0 && ws < count) {
                bf16x8 *dst = obuf + (size_t)((ws & 1) * ks1) * P * 64 + lane;
#pragma unroll
                for (int k = 0; k < KM - 1; ++k)
                    if (k < nfull) put(dst + (k * P) * 64, stage[k]);
                put(dst + (nfull * P) * 64, last);
            }
            if (hw >= 0 && hw < count) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) put(&hin_lds[hw & 1][ks][0][lane], hstage[ks]);
            }
            if (ls >= 0 && ls < count) {
                const int row = item_row(ls);
                const float *r = args.obs + (size_t)(row < rows ? row : 0) * D + 8 * q4;
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
            if (hl >= 0 && hl < count) {
                const int row = item_row(hl);
                const int rr = row < rows ? row : 0;
                const bool keep = !(args.reset && args.reset[rr / N]);
                const float *r = args.h_in + (size_t)rr * H + 4 * q4;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const f32x4 a = *reinterpret_cast<const f32x4 *>(r + 32 * ks);
                    const f32x4 b = *reinterpret_cast<const f32x4 *>(r + 32 * ks + 16);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        hstage[ks][i] = keep ? a[i] : 0.0f;
                        hstage[ks][4 + i] = keep ? b[i] : 0.0f;
                    }
                }
            }
            lds_barrier();
        }
    } else {
        // ---------------------------------------------------------------- fc1 wave
        constexpr int NBF = Sh::NBF, KM = Sh::kKs1Max;
        const int f = wave - Sh::kFc1;
        WFrag<P> w1[NBF][KM];
#pragma unroll
        for (int j = 0; j < NBF; ++j)
#pragma unroll
            for (int ks = 0; ks < KM; ++ks)
                if (ks < ks1) w1[j][ks] = load_wfrag<P>(net.w1_16 + ((size_t)((f * NBF + j) * ks1 + ks) * P) * 64 + lane);
        auto obs_frag = [&](int item, int ks) {
            const bf16x8 *src = obuf + (size_t)(((item & 1) * ks1 + ks) * P) * 64 + lane;
            Frag<P> fr;
            fr.hi = src[0];
            if constexpr (P == 2) fr.lo = src[64];
            return fr;
        };
        // Touching ahead: one 4-byte load per 128 bytes of the observation and hidden-state rows
        // of a later item (see unroll_fused.hip).
        constexpr int kTouchAhead = 4, TLO = (KM * 32 + 127) / 128, TL = TLO + 1;
        int touch_off[TLO];
#pragma unroll
        for (int j = 0; j < TLO; ++j) touch_off[j] = min(32 * (4 * j + q4), D - 1);
        const int touch_off_h = min(32 * q4, H - 1);
        uint32_t touched[kTouchAhead][TL] = {};
        auto touch = [&](uint32_t (&set)[TL], int s) {
            const int row = item_row(s + 3 + kTouchAhead);
            const size_t rr = row < rows ? row : 0;
            const float *r = args.obs + rr * D;
#pragma unroll
            for (int j = 0; j < TL; ++j) asm volatile("" ::"v"(set[j]));
#pragma unroll
            for (int j = 0; j < TLO; ++j) set[j] = __builtin_bit_cast(uint32_t, r[touch_off[j]]);
            set[TLO] = __builtin_bit_cast(uint32_t, args.h_in[rr * H + touch_off_h]);
        };
        auto fc1_step = [&](int s) {
            const int item = s + 1;
            if (item >= 0 && item < count) {
                const int row = item_row(item);
                const int n = (row < rows ? row : 0) % N;
                f32x4 b1v[NBF];
#pragma unroll
                for (int j = 0; j < NBF; ++j) b1v[j] = load_feature4(net.bias1 + (size_t)n * H, f * NBF + j, q4);
                f32x4 acc[NBF];
#pragma unroll
                for (int j = 0; j < NBF; ++j)
#pragma unroll
                    for (int r = 0; r < 4; ++r) acc[j][r] = 0.0f;
                Frag<P> bq[3];
                bq[0] = obs_frag(item, 0);
                bq[1] = obs_frag(item, min(1, ks1 - 1));
#pragma unroll
                for (int ks = 0; ks < KM; ++ks)
                    if (ks < ks1) {
                        bq[(ks + 2) % 3] = obs_frag(item, min(ks + 2, ks1 - 1));
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
                    x_lds[item & 1][f * (NBF / 2) + jj][0][lane] = fr.hi;
                    if constexpr (P == 2) x_lds[item & 1][f * (NBF / 2) + jj][1][lane] = fr.lo;
                }
            }
            lds_barrier();
        };
        int s = -LEAD;
        if (f == 0) {
            static_assert(kTouchAhead == 4, "the loop is unrolled over the register sets");
            for (; s + 3 <= count; s += 4) {
                touch(touched[0], s);     fc1_step(s);
                touch(touched[1], s + 1); fc1_step(s + 1);
                touch(touched[2], s + 2); fc1_step(s + 2);
                touch(touched[3], s + 3); fc1_step(s + 3);
            }
        }
        for (; s <= count; ++s) fc1_step(s);
    }
}

// ------------------------------------------------------------------------------------------ host side
namespace {

template <int H, int P>
hipError_t act_dispatch(const ActFusedArgs &a, hipStream_t stream)
{
    using Sh = Fused16<H, P>;
    const int tiles = (a.rows + 15) / 16;
    const dim3 grid((unsigned)((tiles + a.tiles_per_group - 1) / a.tiles_per_group)), block(fused_threads(H));
    const size_t lds = Sh::lds_bytes_act((a.net.D + 31) / 32);
#define MARL_ACTF(ABLK)                                                                                             \
    do {                                                                                                            \
        auto kernel = act_fused_kernel<H, P, ABLK>;                                                                 \
        hipError_t err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),                               \
                                             hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                 \
        if (err != hipSuccess) return err;                                                                          \
        hipLaunchKernelGGL(kernel, grid, block, lds, stream, a);                                                    \
    } while (0)
    switch ((a.net.A + 15) / 16) {
    case 1: MARL_ACTF(1); break;
    case 2: MARL_ACTF(2); break;
    case 3: MARL_ACTF(3); break;
    case 4: MARL_ACTF(4); break;
    default: return hipErrorInvalidValue;
    }
#undef MARL_ACTF
    return hipGetLastError();
}

template <int H, int P> bool fits_act(const NetFrags &net)
{
    const int ks1 = (net.D + 31) / 32;
    return ks1 <= Fused16<H, P>::kKs1Max && Fused16<H, P>::lds_bytes_act(ks1) <= (size_t)kLdsLimit;
}

}  // namespace

bool act_fused_fits(const NetFrags &net)
{
    if (net.A > 64) return false;
    if (net.H == 64 && net.planes == 2) return fits_act<64, 2>(net);
    if (net.H == 64 && net.planes == 1) return fits_act<64, 1>(net);
    if (net.H == 128 && net.planes == 1) return fits_act<128, 1>(net);
    return false;
}

hipError_t launch_act_fused(const NetFrags &net, int E, int n_groups_hint, const float *obs, const uint8_t *avail,
                            const float *h_in, const uint8_t *reset, const int32_t *step_t, float epsilon,
                            uint64_t seed, float *h_out, int32_t *action, float *q_out, hipStream_t stream)
{
    ActFusedArgs a{};
    a.net = net;
    a.rows = E * net.N;
    const int tiles = (a.rows + 15) / 16;
    const int groups = n_groups_hint > 0 ? n_groups_hint : 256;       // one workgroup per compute unit
    a.tiles_per_group = (tiles + groups - 1) / groups;
    a.obs = obs; a.avail = avail; a.h_in = h_in; a.reset = reset; a.step_t = step_t;
    a.epsilon = epsilon; a.seed = seed; a.h_out = h_out; a.action = action; a.q_out = q_out;
    if (net.H == 64 && net.planes == 2) return act_dispatch<64, 2>(a, stream);
    if (net.H == 64 && net.planes == 1) return act_dispatch<64, 1>(a, stream);
    if (net.H == 128 && net.planes == 1) return act_dispatch<128, 1>(a, stream);
    return hipErrorInvalidValue;
}

}  // namespace marl
