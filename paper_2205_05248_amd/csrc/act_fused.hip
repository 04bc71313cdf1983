// Fused decision-step kernel for gfx950 on tiles of 16 (env, agent) rows.
//
// Same machine as the fused unroll (unroll_fused.hip): every weight stays on chip (W_hh, W1, W2 in
// registers, W_ih in LDS) and the work of a tile is a pipeline over wavefront roles that meet at
// one LDS-only barrier per step.  Here the pipeline runs over the workgroup's *tiles* instead of
// over the slots of an episode: a workgroup owns a run of consecutive tiles, and in the step in
// which the GRU handles item k (the k-th tile of the run)
//
//   loader wave    writes the observations of item k+2 to LDS as bf16 operand fragments and asks
//                  for those of item k+4; it also owns the choice of action apart from the
//                  argmax: availability of item k -> slot masks for the epilogue, and once four
//                  items have their greedy action (or the run ends) the epsilon-greedy draws
//                  for their 64 rows at once and the action store;
//   fc1 waves      x = ReLU(W1 o + b1[agent]) for item k+1;
//   compute waves  item k of the GRU: W_ih x + W_hh h + b for their hidden units, gates, new hidden
//                  state to global memory (fp32) and to LDS (operand form);
//   epilogue wave  item k-1: fc2, Q store, masked argmax (greedy action -> LDS); it also feeds the
//                  incoming hidden state: item k+1 goes to LDS (operand fragments for the
//                  product, fp32 for the blend), item k+3 is asked for.
//
// Every input is read once from HBM and nothing of it is reused, so the whole job is hiding the
// latency of a first touch (a few microseconds under load, longer than a step): each wave that
// reads global memory keeps two items in flight in two register sets, indexed by the parity of the
// item, with the step loop unrolled twice so that the sets never move and a wait covers only the
// loads issued two steps earlier.  The first two items are asked for before the weights are
// loaded.  Nothing depends on the previous item, so the steps are pure throughput; the per-launch
// cost of loading the weights (once per workgroup) is amortised over the run of tiles.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "fused16_roles.h"

namespace marl {

struct ActFusedArgs {
    NetFrags net;
    int rows;                   // rows to serve: (listed) environments x agents
    const int32_t *env_index;   // indexed call: the environments to serve, in any order (entries clamped into 0 .. n_envs - 1)
    int n_envs;                 // environments the arrays hold
    uint32_t n_magic;           // ceil(2^32 / N): floor(p / N) = high word of p * n_magic for p < 2^26 (N >= 2)
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

// Availability bits of the whole row (bit a = action a) from the four lanes' slot masks.
template <int AB>
__device__ __forceinline__ uint64_t row_avail_bits16(uint32_t slots, int q)
{
    uint64_t bits = 0;
#pragma unroll
    for (int ab = 0; ab < AB; ++ab) bits |= (uint64_t)((slots >> (4 * ab)) & 0xFu) << (16 * ab + 4 * q);
    return ((uint64_t)or_quarters((uint32_t)(bits >> 32)) << 32) | or_quarters((uint32_t)bits);
}

constexpr int kActLead = 2;          // steps before item 0 enters the GRU
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// IDX: the rows to serve are those of a list of environments; position p of the list's rows maps to row
// env_index[p / N] N + p % N of the arrays, which every load and store is addressed by.
template <int H, int P, int AB, bool IDX>
__global__ __launch_bounds__(fused_threads(H), 2) void act_fused_kernel(const ActFusedArgs args)
{
    using Sh = Fused16<H, P>;
    constexpr int FBK = Sh::FBK, KS = Sh::KS, LEAD = kActLead;
    static_assert(LEAD % 2 == 0, "register sets are indexed by the parity of the step");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    typedef bf16x8 (*FragBuf)[KS][P][64];
    typedef f32x4 (*StateBuf)[FBK][64];
    const NetFrags &net = args.net;
    const int N = net.N, D = net.D, A = net.A;
    const int ks1 = (D + 31) / 32;
    const FragBuf h_lds = reinterpret_cast<FragBuf>(lds + Sh::oH);                   // new hidden state, compute -> epilogue
    const FragBuf x_lds = reinterpret_cast<FragBuf>(lds + Sh::oX);
    const FragBuf hin_lds = reinterpret_cast<FragBuf>(lds + Sh::hin_offset(ks1));    // old hidden state as operand
    const StateBuf hf_lds = reinterpret_cast<StateBuf>(lds + Sh::hf_offset(ks1));    // old hidden state in fp32, by feature block
    uint32_t (*const slots_lds)[64] = reinterpret_cast<uint32_t (*)[64]>(lds + Sh::slots_offset(ks1));
    struct RowChoice { uint32_t bits_lo, bits_hi; int step; };                       // 12 bytes
    RowChoice (*const choice_lds)[16] = reinterpret_cast<RowChoice (*)[16]>(lds + Sh::choice_offset(ks1));
    uint8_t (*const greedy_lds)[16] = reinterpret_cast<uint8_t (*)[16]>(lds + Sh::greedy_offset(ks1));
    bf16x8 *const obuf = reinterpret_cast<bf16x8 *>(lds + Sh::oObs);
    bf16x8 *const wih_lds = reinterpret_cast<bf16x8 *>(lds + Sh::oWih);

    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rows = args.rows;
    const int tiles = (rows + 15) / 16;
    const int first = blockIdx.x * args.tiles_per_group;
    const int count = min(args.tiles_per_group, tiles - first);       // >= 1 by construction of the grid
    const int last = count + 1;                                       // the last step
    // item k (0 <= k < count) is tile first + k; items past the run re-use its last tile (reads only),
    // rows past the end row 0
    auto item_row = [&](int k) { return (first + min(max(k, 0), count - 1)) * 16 + c; };       // position among the rows to serve
    // A position p is agent p % N of the p / N-th environment served; the division is a multiplication by a
    // constant of the launch.  The indexed call then looks the environment up in the list: a global load, which a
    // wave issues one step before it needs the result (EnvAhead) so that no address ever waits for it.
    struct Served { int env, n; };
    auto served_at = [&](int k) {                                                              // item k -> (p / N, p % N)
        int pos = item_row(k);
        pos = pos < rows ? pos : 0;
        const int listed = N == 1 ? pos : (int)__umulhi((uint32_t)pos, args.n_magic);
        return Served{listed, pos - listed * N};
    };
    auto env_of = [&](int k) {                                                                 // the environment of item k's row
        const int listed = served_at(k).env;
        if constexpr (IDX) return min(max(args.env_index[listed], 0), args.n_envs - 1);
        else return listed;
    };
    auto row_in = [&](int env, int k) { return env * N + served_at(k).n; };                    // row of the arrays
    struct EnvAhead {                      // env_of(item) for the item of the next call, asked for during this one
        int next;
        __device__ __forceinline__ int take(int upcoming) { const int now = next; next = upcoming; return now; }
    };
    // Steps run s = -LEAD .. count + 1, one barrier at the end of each: LEAD + count + 2 barriers per wave.
    // Step s = s0 + u of the unrolled loops has the parity of u.

    auto stage_wih = [&]() {             // every wave's share of W_ih -> LDS
        constexpr int kVecs = 3 * FBK * KS * P * 64, kRounds = kVecs / fused_threads(H);
        static_assert(kVecs % fused_threads(H) == 0, "whole rounds");
        // every workgroup copies the same bytes at the same time: each starts at another round, so that at any
        // moment the compute units ask different L2 channels
        const int first_round = blockIdx.x % kRounds;
#pragma unroll
        for (int r = 0; r < kRounds; ++r) {
            int round = first_round + r;
            round = round >= kRounds ? round - kRounds : round;
            const int i = round * fused_threads(H) + threadIdx.x;
            wih_lds[i] = net.wih_16[i];
        }
    };

    if (wave < Sh::NC) {
        // ---------------------------------------------------------------- compute wave
        constexpr int NBC = Sh::NBC;
        const int w = wave;
        stage_wih();
        GruWave<H, P> gru;
        gru.load(net, w, lane, q4);
        if (w == 0) GruWave<H, P>::stage_gate_biases(lds, net, lane);
        gru.settle_weights();
        EnvAhead ahead{env_of(0)};
        for (int i = 0; i < LEAD; ++i) lds_barrier();
        for (int s = 0; s <= last; ++s) {
            const int env = ahead.take(env_of(s + 1));
            if (s < count) {
                const int cur = s & 1;
                const bool valid = item_row(s) < rows;
                const int row = row_in(env, s);
                f32x4 hv[NBC];           // this wave's own units of the old state in fp32, for the blend
#pragma unroll
                for (int j = 0; j < NBC; ++j) hv[j] = hf_lds[cur][NBC * w + j][lane];
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
        // Its steps are straight-line code with the same memory operations in every step, so
        // that a wait on a register set counts exactly the operations issued since and covers
        // nothing younger: loads of items outside the run read clamped rows, stores of items
        // outside the run (and of rows past the end, and of Q when it is not wanted) carry an
        // offset outside their buffer descriptor and are dropped by the hardware.
        // Hidden state: the operand of k-step ks wants features 32 ks + 16 (idx / 4) + 4 q + idx % 4,
        // i.e. two aligned groups of four floats, which are also the lane's share of feature
        // blocks 2 ks and 2 ks + 1.
        struct StateIn { f32x4 a[KS], b[KS]; uint32_t flag; };
        const bool has_reset = args.reset != nullptr;
        // without reset flags the byte is read from step_t instead and ignored
        const uint8_t *const flag_src = has_reset ? args.reset : reinterpret_cast<const uint8_t *>(args.step_t);
        auto fetch_state = [&](int k, int env) {
            StateIn st;
            const int rr = row_in(env, k);
            const float *r = args.h_in + (size_t)rr * H + 4 * q4;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                st.a[ks] = *reinterpret_cast<const f32x4 *>(r + 32 * ks);
                st.b[ks] = *reinterpret_cast<const f32x4 *>(r + 32 * ks + 16);
            }
            st.flag = flag_src[env];
            return st;
        };
        StateIn state[2] = {fetch_state(0, env_of(0)), fetch_state(1, env_of(1))};
        EnvAhead state_ahead{env_of(-LEAD + 3)}, out_ahead{env_of(-LEAD - 1)};
        stage_wih();
        float *const b2_lds = reinterpret_cast<float *>(lds + Sh::oB2);
        WFrag<P> w2[AB][KS];
#pragma unroll
        for (int ab = 0; ab < AB; ++ab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) w2[ab][ks] = load_wfrag<P>(net.w2_16 + ((size_t)(ab * KS + ks) * P) * 64 + lane);
        if (lane < 16 * AB) b2_lds[lane] = lane < A ? net.b2[lane] : 0.0f;
#pragma unroll
        for (int ab = 0; ab < AB; ++ab)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) settle(w2[ab][ks]);
        // outputs of this workgroup's run of tiles, addressed by row within the run
        // (indexed call: of the whole array, addressed by array row; the host has checked that it fits 32-bit offsets)
        const int run_rows = min(count * 16, rows - first * 16);
        const __amdgpu_buffer_rsrc_t q_buf = __builtin_amdgcn_make_buffer_rsrc(
            args.q_out + (IDX ? (size_t)0 : (size_t)first * 16 * A), 0,
            args.q_out ? (IDX ? args.n_envs * N : run_rows) * A * 4 : 0, kRawBuffer);
        constexpr uint32_t kDrop = 0xFFFFFFF0u;              // beyond any descriptor
        auto step = [&](auto set, int s) {
            constexpr int p = 1 - decltype(set)::value;      // parity of items s - 1, s + 1, s + 3
            // item s - 1: every LDS read it needs is asked for first (the LDS queue is long while
            // the compute waves stream W_ih through it) and arrives during the work on the state
            const int k = s - 1, cur = k & 1;
            f32x4 qv[AB];
            Frag<P> hb[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                hb[ks].hi = h_lds[cur][ks][0][lane];
                if constexpr (P == 2) hb[ks].lo = h_lds[cur][ks][1][lane];
            }
#pragma unroll
            for (int ab = 0; ab < AB; ++ab) qv[ab] = load_feature4(b2_lds, ab, q4);
            __builtin_amdgcn_sched_barrier(0);
            {   // incoming hidden state of item s + 1 -> LDS, that of item s + 3 asked for
                const int nb = (s + 1) & 1;
                const bool keep = !(has_reset && (state[p].flag & 0xFFu));
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    f32x4 a = state[p].a[ks], b = state[p].b[ks];
                    float v[8];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        a[i] = keep ? a[i] : 0.0f;
                        b[i] = keep ? b[i] : 0.0f;
                        v[i] = a[i];
                        v[4 + i] = b[i];
                    }
                    ObsStage<H, P>::put(&hin_lds[nb][ks][0][lane], v);
                    hf_lds[nb][2 * ks][lane] = a;
                    hf_lds[nb][2 * ks + 1][lane] = b;
                }
                state[p] = fetch_state(s + 3, state_ahead.take(env_of(s + 4)));
            }
            __builtin_amdgcn_sched_barrier(0);
            {   // item s - 1: Q, mask, choice
                const int out_env = out_ahead.take(env_of(s));           // item k of this step; item s - 1 + 1 for the next
                const int lr = IDX ? row_in(out_env, k) : k * 16 + c;    // row within the run (indexed call: of the array)
                // (the run-relative addresses of the dense call fall outside the descriptor for items past the run)
                uint32_t dead = k >= 0 && (!IDX || (k < count && item_row(k) < rows)) ? 0u : kDrop;      // in a vector register: the step must not fork on it
                asm volatile("" : "+v"(dead));
#pragma unroll
                for (int ks = 0; ks < KS; ++ks)
                    {
                        f32x4 *accs[AB];
                        const WFrag<P> *wf[AB];
#pragma unroll
                        for (int ab = 0; ab < AB; ++ab) {
                            accs[ab] = &qv[ab];
                            wf[ab] = &w2[ab][ks];
                        }
                        mma16_across<P, AB>(accs, wf, hb[ks]);
                    }
                if ((A & 3) == 0) {                          // a lane's four actions of a block: 16 aligned bytes
#pragma unroll
                    for (int ab = 0; ab < AB; ++ab) {
                        const int a = 16 * ab + 4 * q4;
                        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, qv[ab]), q_buf,
                                                               (a < A ? (uint32_t)(lr * A + a) * 4u : kDrop) | dead, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int ab = 0; ab < AB; ++ab)
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const int a = 16 * ab + 4 * q4 + r;
                            const float value = qv[ab][r];
                            __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(value), q_buf,
                                                                  (a < A ? (uint32_t)(lr * A + a) * 4u : kDrop) | dead, 0, 0);
                        }
                }
                const uint32_t slots = slots_lds[cur][lane];     // from the loader, one step ago
                float best_q; int best;
                masked_argmax16<AB>(qv, slots, q4, best_q, best);
                greedy_lds[k & 7][c] = (uint8_t)max(best, 0);    // the four lanes of a row agree
            }
            lds_barrier();
        };
        int s = -LEAD;
        for (; s + 1 <= last; s += 2) {
            step(std::integral_constant<int, 0>{}, s);
            step(std::integral_constant<int, 1>{}, s + 1);
        }
        if (s <= last) step(std::integral_constant<int, 0>{}, s);
    } else if (wave == Sh::kLoader) {
        // ---------------------------------------------------------------- loader wave
        // straight-line steps like the epilogue's; items past the run are read again from its
        // last tile and land in LDS buffers that nobody reads any more
        ObsStage<H, P> st;
        st.init(D, ks1, q4);
        ObsRegs<H, P> regs[2];
        auto obs_row8 = [&](int k, int env) { return args.obs + (size_t)row_in(env, k) * D + 8 * q4; };
        st.load(regs[0], obs_row8(0, env_of(0)));
        st.load(regs[1], obs_row8(1, env_of(1)));
        EnvAhead obs_ahead{env_of(-LEAD + 4)};       // the item whose observations are fetched next, looked up a step early
        stage_wih();
        auto step = [&](auto set, int s) {
            constexpr int u = decltype(set)::value;          // parity of items s, s + 2, s + 4
            st.write(regs[u], obuf + (size_t)((s & 1) * ks1) * P * 64 + lane);
            st.load(regs[u], obs_row8(s + 4, obs_ahead.take(env_of(s + 5))));
            lds_barrier();
        };
        int s = -LEAD;
        for (; s + 1 <= last; s += 2) {
            step(std::integral_constant<int, 0>{}, s);
            step(std::integral_constant<int, 1>{}, s + 1);
        }
        if (s <= last) step(std::integral_constant<int, 0>{}, s);
    } else {
        // ---------------------------------------------------------------- fc1 wave
        // Besides x, each of the two takes one side job of the choice of action off the loader (which is the wave
        // with the most to do in a step): the first the availability of item s (slot masks for the epilogue's
        // argmax, the row's bits and step number for the draw), the second the draw itself.
        const int f = wave - Sh::kFc1;
        stage_wih();
        Fc1Wave<H, P> fc1;
        fc1.load(net, f, ks1, lane);
        fc1.settle_weights(ks1);
        struct ItemIn { uint32_t avail_raw[AB]; int step; };
        auto fetch_item = [&](int k, int env) {
            ItemIn in;
            issue_avail_loads16<AB>(args.avail + (size_t)row_in(env, k) * A, A, q4, in.avail_raw);
            in.step = args.step_t[env];
            return in;
        };
        auto fc1_item = [&](int s) {
            const int item = s + 1;
            if (item >= 0 && item < count) {
                f32x4 b1v[Sh::NBF];
                Fc1Wave<H, P>::load_bias(net, f, served_at(item).n, q4, b1v);
                fc1.step(obuf + (size_t)((item & 1) * ks1) * P * 64, ks1, f, lane, b1v, x_lds[item & 1]);
            }
        };
        if (f == 0) {
            ItemIn in[2] = {fetch_item(0, env_of(0)), fetch_item(1, env_of(1))};
            EnvAhead item_ahead{env_of(-LEAD + 2)};      // the item whose availability is fetched next, looked up a step early
            auto step = [&](auto set, int s) {
                constexpr int u = decltype(set)::value;      // parity of items s, s + 2
                fc1_item(s);
                const uint32_t slots = avail_mask16<AB>(in[u].avail_raw, A, q4, true);
                slots_lds[s & 1][lane] = slots;
                const uint64_t bits = row_avail_bits16<AB>(slots, q4);
                choice_lds[s & 7][c] = {(uint32_t)bits, (uint32_t)(bits >> 32), in[u].step};      // the four lanes of a row agree
                in[u] = fetch_item(s + 2, item_ahead.take(env_of(s + 3)));
                lds_barrier();
            };
            int s = -LEAD;
            for (; s + 1 <= last; s += 2) {
                step(std::integral_constant<int, 0>{}, s);
                step(std::integral_constant<int, 1>{}, s + 1);
            }
            if (s <= last) step(std::integral_constant<int, 0>{}, s);
        } else {
            // actions of this workgroup's run of tiles, addressed by row within the run
            const __amdgpu_buffer_rsrc_t action_buf = __builtin_amdgcn_make_buffer_rsrc(
                args.action + (IDX ? (size_t)0 : (size_t)first * 16), 0,
                (IDX ? args.n_envs * N : min(count * 16, rows - first * 16)) * 4, kRawBuffer);
            constexpr uint32_t kDrop = 0xFFFFFFF0u;          // beyond any descriptor
            auto pick_item = [&](int s) { return ((s - 2) & ~3) + q4; };
            EnvAhead pick_ahead{env_of(pick_item(-LEAD))};   // the item whose action is drawn next, looked up a step early
            for (int s = -LEAD; s <= last; ++s) {
                fc1_item(s);
                // The draw is the same work for one lane or sixty-four, so it waits until four items
                // have their greedy action (or the run ends) and is then made for their 64 rows at
                // once: lane quarter q takes item 4 i + q.  Item s - 2 got its greedy action in the
                // previous step.
                const int k = s - 2;
                int pick = 0;
                uint32_t pick_at = kDrop;
                const int pick_env = pick_ahead.take(env_of(pick_item(s + 1)));
                if ((k & 3) == 3 || k == count - 1) {
                    const int kk = (k & ~3) + q4;
                    const RowChoice ch = choice_lds[kk & 7][c];
                    const int greedy = greedy_lds[kk & 7][c];
                    const int rr = row_in(pick_env, kk);
                    pick = eps_greedy_pick(greedy, ((uint64_t)ch.bits_hi << 32) | ch.bits_lo, args.epsilon, args.seed,
                                           (uint32_t)pick_env, (uint32_t)served_at(kk).n, (uint32_t)ch.step);
                    if constexpr (IDX) pick_at = kk >= 0 && kk <= k && item_row(kk) < rows ? (uint32_t)rr * 4u : kDrop;
                    else pick_at = kk >= 0 && kk <= k ? (uint32_t)(kk * 16 + c) * 4u : kDrop;
                }
                __builtin_amdgcn_raw_buffer_store_b32((uint32_t)pick, action_buf, pick_at, 0, 0);
                lds_barrier();
            }
        }
    }
}

// ------------------------------------------------------------------------------------------ host side
namespace {

template <int H, int P, bool IDX>
hipError_t act_dispatch(const ActFusedArgs &a, hipStream_t stream)
{
    using Sh = Fused16<H, P>;
    const int tiles = (a.rows + 15) / 16;
    const dim3 grid((unsigned)((tiles + a.tiles_per_group - 1) / a.tiles_per_group)), block(fused_threads(H));
    const size_t lds = Sh::lds_bytes_act((a.net.D + 31) / 32);
#define MARL_ACTF(ABLK)                                                                                             \
    do {                                                                                                            \
        auto kernel = act_fused_kernel<H, P, ABLK, IDX>;                                                            \
        hipError_t err = allow_large_lds<act_fused_kernel<H, P, ABLK, IDX>>(kLdsLimit);                             \
        if (err != hipSuccess) return err;                                                                          \
        launch_kernel(kernel, grid, block, lds, stream, a);                                                         \
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
    if (net.A > 64 || net.A < 4) return false;       // availability is read four bytes at a time
    if (net.H == 64 && net.planes == 2) return fits_act<64, 2>(net);
    if (net.H == 64 && net.planes == 1) return fits_act<64, 1>(net);
    if (net.H == 128 && net.planes == 1) return fits_act<128, 1>(net);
    return false;
}

hipError_t launch_act_fused(const NetFrags &net, int E, const int32_t *env_index, int n_listed, int n_groups_hint,
                            const float *obs, const uint8_t *avail,
                            const float *h_in, const uint8_t *reset, const int32_t *step_t, float epsilon,
                            uint64_t seed, float *h_out, int32_t *action, float *q_out, hipStream_t stream)
{
    ActFusedArgs a{};
    a.net = net;
    a.rows = (env_index ? n_listed : E) * net.N;
    a.env_index = env_index;
    a.n_envs = E;
    a.n_magic = net.N == 1 ? 0u : (uint32_t)(((1ull << 32) + net.N - 1) / net.N);
    const int tiles = (a.rows + 15) / 16;
    const int groups = n_groups_hint > 0 ? n_groups_hint : 256;       // one workgroup per compute unit
    a.tiles_per_group = (tiles + groups - 1) / groups;
    a.obs = obs; a.avail = avail; a.h_in = h_in; a.reset = reset; a.step_t = step_t;
    a.epsilon = epsilon; a.seed = seed; a.h_out = h_out; a.action = action; a.q_out = q_out;
#define MARL_GO(HH, PP) return env_index ? act_dispatch<HH, PP, true>(a, stream) : act_dispatch<HH, PP, false>(a, stream)
    if (net.H == 64 && net.planes == 2) MARL_GO(64, 2);
    if (net.H == 64 && net.planes == 1) MARL_GO(64, 1);
    if (net.H == 128 && net.planes == 1) MARL_GO(128, 1);
#undef MARL_GO
    return hipErrorInvalidValue;
}

// The indexed call addresses Q values and actions of the whole arrays with 32-bit byte offsets.
bool act_fused_indexed_fits(const NetFrags &net, int E)
{
    return act_fused_rows_fit(net, E) && (long)E * net.N * net.A * 4 < (1l << 31);
}

// Rows are split into (environment, agent) by a multiplication that is exact below 2^26 rows.
bool act_fused_rows_fit(const NetFrags &net, int E)
{
    return act_fused_fits(net) && (long)E * net.N < (1l << 26);
}

}  // namespace marl
