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

#include "fused16_roles.h"

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
        GruWave<H, P> gru;
        gru.load(net, w, lane, q4);
        if (w == 0) GruWave<H, P>::stage_gate_biases(lds, net, lane);
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
                gru.step(lds, w, lane, q4, hin_lds[cur], x_lds[cur], hv);
#pragma unroll
                for (int j = 0; j < NBC; ++j)
                    if (valid) *reinterpret_cast<f32x4 *>(args.h_out + (size_t)row * H + 16 * (NBC * w + j) + 4 * q4) = hv[j];
                GruWave<H, P>::publish(h_lds[cur], w, lane, hv);         // operand of fc2
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
        // Hidden state: the operand of k-step ks wants features 32 ks + 16 (idx / 4) + 4 q + idx % 4,
        // i.e. two aligned groups of four floats.
        ObsStage<H, P> st;
        st.init(D, ks1, q4);
        float hstage[KS][8];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int i = 0; i < 8; ++i) hstage[ks][i] = 0.0f;
        for (int s = -LEAD; s <= count; ++s) {
            const int ws = s + 2, ls = s + 3;        // observations: item written / loaded in this step
            const int hw = s + 1, hl = s + 2;        // hidden state: one item closer to its use
            if (ws >= 0 && ws < count) st.write(obuf + (size_t)((ws & 1) * ks1) * P * 64 + lane);
            if (hw >= 0 && hw < count) {
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) ObsStage<H, P>::put(&hin_lds[hw & 1][ks][0][lane], hstage[ks]);
            }
            if (ls >= 0 && ls < count) {
                const int row = item_row(ls);
                st.load(args.obs + (size_t)(row < rows ? row : 0) * D + 8 * q4);
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
        const int f = wave - Sh::kFc1;
        Fc1Wave<H, P> fc1;
        fc1.load(net, f, ks1, lane);
        ObsTouch<H, P, 1> tch;                       // one more value per set: the hidden-state row
        tch.init(D, q4);
        const int touch_off_h = min(32 * q4, H - 1);
        auto touch = [&](int c, int s) {             // the item the loader will load kTouchAhead steps from now
            const int row = item_row(s + 3 + kTouchAhead);
            const size_t rr = row < rows ? row : 0;
            tch.consume(c);
            tch.touch(c, args.obs + rr * D);
            tch.set[c][tch.TLO] = __builtin_bit_cast(uint32_t, args.h_in[rr * H + touch_off_h]);
        };
        auto fc1_step = [&](int s) {
            const int item = s + 1;
            if (item >= 0 && item < count) {
                const int row = item_row(item);
                f32x4 b1v[Sh::NBF];
                Fc1Wave<H, P>::load_bias(net, f, (row < rows ? row : 0) % N, q4, b1v);
                fc1.step(obuf + (size_t)((item & 1) * ks1) * P * 64, ks1, f, lane, b1v, x_lds[item & 1]);
            }
            lds_barrier();
        };
        int s = -LEAD;
        if (f == 0) {
            static_assert(kTouchAhead == 4, "the loop is unrolled over the register sets");
            for (; s + 3 <= count; s += 4) {
                touch(0, s);     fc1_step(s);
                touch(1, s + 1); fc1_step(s + 1);
                touch(2, s + 2); fc1_step(s + 2);
                touch(3, s + 3); fc1_step(s + 3);
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
        hipError_t err = allow_large_lds<act_fused_kernel<H, P, ABLK>>(kLdsLimit);                                  \
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
