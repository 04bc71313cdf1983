// gfx950 kernels of the recurrent Q-network on tiles of 32 rows, and their launchers.
//
//   front_kernel<.., ACT>    decision step: every wavefront owns tiles of 32 (env, agent) rows and
//                            runs fc1 -> GRU cell -> fc2 -> mask/argmax/epsilon-greedy without its
//                            activations leaving registers; the weights stream through LDS.
//   front_kernel<.., !ACT>   two-kernel unroll, part 1: fc1 and the input half of the GRU gates for
//                            every (episode, slot, agent); no dependence on the hidden state, so all
//                            B (T+1) N rows run in parallel.  Results go to a scratch buffer in the
//                            accumulator layout of the consumer.
//   recurrent_td_kernel      two-kernel unroll, part 2: one workgroup per 32 (episode, agent) rows
//                            walks the T+1 slots, adds the hidden half of the gates, applies fc2 and
//                            emits q_taken / next_max / td_target.
// The default unroll is the fused kernel of unroll_fused.hip; this pair serves the networks that do
// not fit it.
#include "mfma_tile.h"
#include "stream_layout.h"
#include "recurrent_roles.h"

namespace marl {

// ------------------------------------------------------------------------------------------ front end
// Decision step (ACT) and input projection of the unroll (!ACT) share one kernel.  A workgroup
// of NW wavefronts owns NW tiles of 32 rows; each wavefront keeps its rows' activations in
// registers from layer to layer.  The weights are not read per wavefront from global memory:
// the whole workgroup pulls them through LDS in chunks of kChunkPlanes fragment planes, in the
// order of use fixed by stream_layout.h, double-buffered: while chunk c is consumed, chunk c+1
// sits in registers on its way to the other LDS buffer and chunk c+2 is in flight from L2.
// One LDS-only barrier per chunk.
//
struct FrontArgs {
    NetFrags net[2];            // ACT: net[0]; projection: online, target (blockIdx.y)
    // decision step
    int rows;                   // rows to process: (listed) environments x agents
    const int32_t *env_index;   // null: environments 0 .. rows/N - 1; else the environments to serve, in any order
    int n_envs;                 // environments the arrays hold (listed indices are clamped into it)
    const float *obs;
    const uint8_t *avail;
    const float *h_in;
    const uint8_t *reset;
    const int32_t *step_t;
    float epsilon;
    uint64_t seed;
    float *h_out;
    int32_t *action;
    float *q_out;
    // input projection
    char *gi[2];
    int B, T;
    const int32_t *episode_index;   // null, or the pool episode of each batch position
    int pool_episodes;
    unsigned nets;              // 1 or 2
};

// Four wavefronts per workgroup, one per SIMD with the whole register file, each owning NC column
// blocks of 32 rows: a weight fragment read from LDS then feeds NC MFMAs, which keeps LDS reads
// below the matrix pipe's appetite.  NC = 2 whenever two blocks' operands fit in 512 registers.
constexpr int kFrontWaves = 4;
constexpr int kFrontThreads = 64 * kFrontWaves;
constexpr int kFrontStage = kChunkVecs / kFrontThreads;          // 16-byte vectors per thread and chunk
constexpr int front_col_blocks(int H, int P) { return (H * P <= 128) ? 2 : 1; }

template <int H, int P, int MB2, bool ACT>
__global__ __launch_bounds__(kFrontThreads, 1) void front_kernel(const FrontArgs args)
{
    constexpr int MB = H / 32, FB = H / 32, KCH = H / 16;
    constexpr int NC = front_col_blocks(H, P), NT = kFrontThreads, STG = kFrontStage;
    constexpr StreamDims SD = stream_dims(H, P, MB2);
    constexpr int OB = 3;                             // observation k-steps fetched ahead as one block
    constexpr int SUB = SD.kpc / OB;
    static_assert(SD.kpc % OB == 0, "fc1 chunk must hold whole observation blocks");
    __shared__ bf16x8 wbuf[2][kChunkVecs];

    const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, col = lane & 31;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // projection: the two networks' workgroups alternate in launch order, so the second one to
    // read an observation tile finds it in cache
    const int net_id = ACT ? 0 : (int)(blockIdx.x % args.nets);
    const unsigned group_id = ACT ? blockIdx.x : blockIdx.x / args.nets;
    const NetFrags &net = args.net[net_id];
    const int N = net.N, D = net.D, A = net.A;

    // ---- which rows this wavefront owns: column block c holds rows row[c] = 32 (tile + c) + col
    bool valid[NC];
    int row[NC], n[NC];
    const float *obs_row[NC];
    [[maybe_unused]] int e[NC];
    [[maybe_unused]] char *gi_dst[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        if constexpr (ACT) {
            // position in the list of rows to serve -> (environment, agent) -> row of the arrays
            const int at = ((group_id * kFrontWaves + wave) * NC + c) * 32 + col;
            valid[c] = at < args.rows;
            const int listed = valid[c] ? at / N : 0;
            n[c] = valid[c] ? at % N : 0;
            e[c] = args.env_index ? min(max(args.env_index[listed], 0), args.n_envs - 1) : listed;
            row[c] = valid[c] ? e[c] * N + n[c] : 0;                         // positions past the end read row 0, unused
            obs_row[c] = args.obs + (size_t)row[c] * D;
        } else {
            const int rows = args.B * N, S = args.T + 1, ntiles = (rows + 31) / 32, ngroups = (ntiles + NC - 1) / NC;
            const long work = (long)group_id * kFrontWaves + wave;        // (group of NC row tiles, slot)
            const bool in_range = work < (long)ngroups * S;
            const int rt = (in_range ? (int)(work / S) : 0) * NC + c, t = in_range ? (int)(work % S) : 0;
            const bool tile_ok = in_range && rt < ntiles;
            row[c] = rt * 32 + col;
            valid[c] = tile_ok && row[c] < rows;
            const int b = valid[c] ? row[c] / N : 0;
            const int bi = args.episode_index ? min(max(args.episode_index[b], 0), args.pool_episodes - 1) : b;
            n[c] = valid[c] ? row[c] % N : 0;
            obs_row[c] = args.obs + (valid[c] ? (((size_t)bi * S + t) * N + n[c]) * D : 0);
            gi_dst[c] = tile_ok ? args.gi[net_id] + ((size_t)rt * S + t) * (3 * FB * GiLayout<P>::kBlockBytes) : nullptr;
        }
    }

    // ---- weight pipeline
    const bf16x8 *stream = ACT ? net.act_stream : net.proj_stream;
    const int total = ACT ? net.act_chunks : net.proj_chunks;
    bf16x8 stage[STG];
    int chunk = 0;
    auto fetch = [&](int c) {
        if (c < total) {
            const bf16x8 *src = stream + (size_t)c * kChunkVecs + tid;
#pragma unroll
            for (int i = 0; i < STG; ++i) stage[i] = src[i * NT];
        }
    };
    auto commit = [&](int c) {
        if (c < total) {
            bf16x8 *dst = &wbuf[c & 1][tid];
#pragma unroll
            for (int i = 0; i < STG; ++i) dst[i * NT] = stage[i];
        }
    };
    auto advance = [&]() {          // done with chunk `chunk`: publish the next one, start the one after
        commit(chunk + 1);
        fetch(chunk + 2);
        lds_barrier();
        ++chunk;
    };
    fetch(0);

    // ---- decision step: issue the rows' other inputs early
    [[maybe_unused]] bool keep_h[NC];
    [[maybe_unused]] const float *h_row[NC];
    [[maybe_unused]] const uint8_t *avail_row[NC];
    [[maybe_unused]] uint32_t avail_raw[NC][MB2 * 4];
    [[maybe_unused]] Frag<P> hf[NC][KCH];
    if constexpr (ACT) {
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            keep_h[c] = valid[c] && !(args.reset && args.reset[e[c]]);
            h_row[c] = args.h_in + (size_t)row[c] * H;
            avail_row[c] = args.avail + (valid[c] ? (size_t)row[c] * A : 0);
            if (A >= 4) issue_avail_loads<MB2>(avail_row[c], A, lane, avail_raw[c]);      // consumed after fc2
#pragma unroll
            for (int b = 0; b < FB; ++b) {                  // hidden state as operand fragments
                f32x16 hv;
                if (keep_h[c]) hv = load_feature_block(h_row[c], b, g);
                else
#pragma unroll
                    for (int r = 0; r < 16; ++r) hv[r] = 0.0f;
                hf[c][2 * b] = frag_of_half<P>(hv, 0);
                hf[c][2 * b + 1] = frag_of_half<P>(hv, 1);
            }
        }
    }

    // ---- fc1 + ReLU
    bool vec4 = (D % 4) == 0;
#pragma unroll
    for (int c = 0; c < NC; ++c) vec4 = vec4 && (reinterpret_cast<uintptr_t>(obs_row[c]) & 15u) == 0;
    float cur[NC][OB][8], nxt[NC][OB][8];
    f32x16 acc[NC][MB];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
#pragma unroll
        for (int kk = 0; kk < OB; ++kk) load_obs_chunk(obs_row[c], D, vec4, kk, g, cur[c][kk]);
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) acc[c][mb] = load_feature_block(net.bias1 + (size_t)n[c] * H, mb, g);
    }
    commit(0);
    fetch(1);
    lds_barrier();

    for (int c1 = 0; c1 < net.nc1; ++c1) {
        const bf16x8 *wb = &wbuf[chunk & 1][lane];
#pragma unroll
        for (int s = 0; s < SUB; ++s) {
            const int next_block = c1 * SUB + s + 1;
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int kk = 0; kk < OB; ++kk) load_obs_chunk(obs_row[c], D, vec4, next_block * OB + kk, g, nxt[c][kk]);
#pragma unroll
            for (int kk = 0; kk < OB; ++kk) {
                Frag<P> bfrag[NC];
#pragma unroll
                for (int c = 0; c < NC; ++c) bfrag[c] = to_frag<P>(cur[c][kk]);
#pragma unroll
                for (int mb = 0; mb < MB; ++mb) {
                    const WFrag<P> w = load_wfrag<P>(wb + (((s * OB + kk) * MB + mb) * P) * 64);
#pragma unroll
                    for (int c = 0; c < NC; ++c) mma<P>(acc[c][mb], w, bfrag[c]);
                }
            }
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int kk = 0; kk < OB; ++kk)
#pragma unroll
                    for (int i = 0; i < 8; ++i) cur[c][kk][i] = nxt[c][kk][i];
        }
        advance();
    }
    Frag<P> x[NC][KCH];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb) {
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][mb][r] = fmaxf(acc[c][mb][r], 0.0f);
            x[c][2 * mb] = frag_of_half<P>(acc[c][mb], 0);
            x[c][2 * mb + 1] = frag_of_half<P>(acc[c][mb], 1);
        }

    // ---- GRU
    [[maybe_unused]] Frag<P> hq[NC][KCH];
#pragma unroll
    for (int fb = 0; fb < FB; ++fb) {
        f32x16 ar[NC], az[NC], ain[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            ar[c] = load_feature_block(net.bias_r, fb, g);
            az[c] = load_feature_block(net.bias_z, fb, g);
            ain[c] = load_feature_block(net.bias_in, fb, g);
        }
        if constexpr (ACT) {
            f32x16 ahn[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) ahn[c] = load_feature_block(net.bias_hn, fb, g);
#pragma unroll
            for (int cc = 0; cc < SD.cpf; ++cc) {
                const bf16x8 *wb = &wbuf[chunk & 1][lane];
#pragma unroll
                for (int kk = 0; kk < SD.kpg; ++kk) {
                    const int kc = cc * SD.kpg + kk;
                    const bf16x8 *m = wb + (kk * 6 * P) * 64;
                    const WFrag<P> wir = load_wfrag<P>(m + 0 * P * 64), wiz = load_wfrag<P>(m + 1 * P * 64);
                    const WFrag<P> win = load_wfrag<P>(m + 2 * P * 64), whr = load_wfrag<P>(m + 3 * P * 64);
                    const WFrag<P> whz = load_wfrag<P>(m + 4 * P * 64), whn = load_wfrag<P>(m + 5 * P * 64);
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        mma<P>(ar[c], wir, x[c][kc]);
                        mma<P>(az[c], wiz, x[c][kc]);
                        mma<P>(ain[c], win, x[c][kc]);
                        mma<P>(ar[c], whr, hf[c][kc]);
                        mma<P>(az[c], whz, hf[c][kc]);
                        mma<P>(ahn[c], whn, hf[c][kc]);
                    }
                }
                advance();
            }
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                f32x16 hv;                                       // exact fp32 hidden state for the blend
                if (keep_h[c]) hv = load_feature_block(h_row[c], fb, g);
                else
#pragma unroll
                    for (int r = 0; r < 16; ++r) hv[r] = 0.0f;
                const f32x16 hn = gru_blend(ar[c], az[c], ain[c], ahn[c], hv);
                if (valid[c]) store_feature_block(args.h_out + (size_t)row[c] * H, fb, g, hn);
                hq[c][2 * fb] = frag_of_half<P>(hn, 0);
                hq[c][2 * fb + 1] = frag_of_half<P>(hn, 1);
            }
        } else {
#pragma unroll
            for (int cc = 0; cc < SD.cpj; ++cc) {
                const bf16x8 *wb = &wbuf[chunk & 1][lane];
#pragma unroll
                for (int kk = 0; kk < SD.kpj; ++kk) {
                    const int kc = cc * SD.kpj + kk;
                    const bf16x8 *m = wb + (kk * 3 * P) * 64;
                    const WFrag<P> wir = load_wfrag<P>(m + 0 * P * 64), wiz = load_wfrag<P>(m + 1 * P * 64);
                    const WFrag<P> win = load_wfrag<P>(m + 2 * P * 64);
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        mma<P>(ar[c], wir, x[c][kc]);
                        mma<P>(az[c], wiz, x[c][kc]);
                        mma<P>(ain[c], win, x[c][kc]);
                    }
                }
                advance();
            }
#pragma unroll
            for (int c = 0; c < NC; ++c)
                if (gi_dst[c]) {
                    store_gi_block<P>(gi_dst[c] + (0 * FB + fb) * GiLayout<P>::kBlockBytes, lane, ar[c]);
                    store_gi_block<P>(gi_dst[c] + (1 * FB + fb) * GiLayout<P>::kBlockBytes, lane, az[c]);
                    store_gi_block<P>(gi_dst[c] + (2 * FB + fb) * GiLayout<P>::kBlockBytes, lane, ain[c]);
                }
        }
    }

    // ---- fc2, mask, action
    if constexpr (ACT) {
        f32x16 q[NC][MB2];
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int mb = 0; mb < MB2; ++mb) q[c][mb] = load_feature_block(net.b2, mb, g);
#pragma unroll
        for (int cf = 0; cf < SD.ncf; ++cf) {
            const bf16x8 *wb = &wbuf[chunk & 1][lane];
#pragma unroll
            for (int kk = 0; kk < SD.kpf; ++kk) {
                const int kc = cf * SD.kpf + kk;
                if (kc < KCH) {
#pragma unroll
                    for (int mb = 0; mb < MB2; ++mb) {
                        const WFrag<P> w = load_wfrag<P>(wb + ((kk * MB2 + mb) * P) * 64);
#pragma unroll
                        for (int c = 0; c < NC; ++c) mma<P>(q[c][mb], w, hq[c][kc]);
                    }
                }
            }
            advance();
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            if (args.q_out && valid[c]) store_q_row<MB2>(args.q_out + (size_t)row[c] * A, q[c], A, lane);
            const uint32_t slots = A >= 4 ? avail_mask_from_raw<MB2>(avail_raw[c], A, lane, valid[c])
                                          : avail_mask_small(avail_row[c], A, lane, valid[c]);
            float best_q; int best;
            masked_argmax_slots<MB2>(q[c], slots, lane, best_q, best);
            const uint64_t bits = row_avail_bits<MB2>(slots, lane);
            if (valid[c] && g == 0) {
                if (best < 0) best = 0;
                args.action[row[c]] = eps_greedy_pick(best, bits, args.epsilon, args.seed, (uint32_t)e[c],
                                                      (uint32_t)n[c], (uint32_t)args.step_t[e[c]]);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------ unroll, part 2
// One workgroup per 32 (episode, agent) rows and network; its wavefronts have three roles:
//   compute wave w (w < H/32)  owns hidden units 32w .. 32w+31: its slice of W_hh stays in
//                              registers for the whole episode; each slot it reads the full
//                              hidden state (operand form) and its gate inputs from LDS, does
//                              the hidden projection, the gates, and publishes its 32 new units.
//   epilogue wave              one slot behind: fc2 on the published hidden state (W2 in
//                              registers), then q_taken / masked max / TD target.
//   prefetch waves             copy the gate inputs of the next slots from the scratch buffer
//                              into LDS, one slot ahead in LDS and one more in registers.
// All waves meet at one barrier per slot; LDS buffers are double-buffered across it.
//
// grid = (row tiles, networks).  blockIdx.y = 0: online network, emits q_taken (and q_all);
// blockIdx.y = 1 (distinct target network): emits next_max and td_target.  With one network a
// single pass emits everything.
constexpr int recurrent_waves(int H) { return H / 32 + 1 + (H == 128 ? 3 : 1); }
template <int H, int P> struct RecurrentShape {
    static constexpr int kCompute = H / 32;
    static constexpr int kPrefetch = H == 128 ? 3 : 1;
    static constexpr int kWaves = kCompute + 1 + kPrefetch;
    static constexpr int kGiBytes = 3 * (H / 32) * GiLayout<P>::kBlockBytes;   // per (tile, slot)
    static constexpr int kVecPerLane = kGiBytes / 16 / 64 / kPrefetch;         // 16-byte vectors per prefetch lane and slot
    static_assert(kVecPerLane * 16 * 64 * kPrefetch == kGiBytes, "record must split evenly over the prefetch lanes");
};

template <int H, int P, int MB2, bool QALL>
__global__ __launch_bounds__(64 * recurrent_waves(H), 2) void recurrent_td_kernel(
    NetFrags online, NetFrags target, const char *__restrict__ gi_online, const char *__restrict__ gi_target,
    int two_nets, int B, int T, const int32_t *__restrict__ episode_index, int pool_episodes,
    const uint8_t *__restrict__ avail, const int32_t *__restrict__ actions,
    const float *__restrict__ reward, const uint8_t *__restrict__ terminated, const uint8_t *__restrict__ filled,
    float gamma, float *__restrict__ q_taken, float *__restrict__ next_max, float *__restrict__ td_target,
    float *__restrict__ q_all, int mode, int32_t *__restrict__ next_action)
{
    using Shape = RecurrentShape<H, P>;
    constexpr int KCH = H / 16;
    __shared__ __attribute__((aligned(16))) char gi_lds[2][Shape::kGiBytes];
    __shared__ bf16x8 h_lds[2][KCH][P][64];
    __shared__ __attribute__((aligned(16))) float b2_lds[32 * MB2];

    const bool is_target = blockIdx.y == 1;
    const NetFrags &net = is_target ? target : online;
    const char *__restrict__ gi = is_target ? gi_target : gi_online;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int S = T + 1;
    const int rt = blockIdx.x;
    const char *gi_tile = gi + (size_t)rt * S * Shape::kGiBytes;

    if (wave < Shape::kCompute) {
        compute_role<H, P>(net, wave, lane, T, 1, &gi_lds[0][0], h_lds);
    } else if (wave == Shape::kCompute) {
        const TdArrays td{episode_index, pool_episodes, avail, actions, reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all,
                          mode, next_action};
        epilogue_role<H, P, MB2, QALL>(net, td, !is_target, is_target || !two_nets, rt, lane, B, T, 1, h_lds, b2_lds);
    } else {
        // ---------------------------------------------------------------- prefetch wave
        constexpr int V = Shape::kVecPerLane;
        const int p = wave - Shape::kCompute - 1;
        const int base = (p * V * 64 + lane) * 16;                       // byte offset of this lane's first vector
        f32x4 stage[V];
        auto fetch = [&](int slot) {
            const char *src = gi_tile + (size_t)slot * Shape::kGiBytes + base;
#pragma unroll
            for (int i = 0; i < V; ++i) stage[i] = *reinterpret_cast<const f32x4 *>(src + i * 1024);
        };
        auto publish = [&](int buf) {
#pragma unroll
            for (int i = 0; i < V; ++i) *reinterpret_cast<f32x4 *>(&gi_lds[buf][base + i * 1024]) = stage[i];
        };
        fetch(0);
        publish(0);
        if (T >= 1) fetch(1);
        lds_barrier();
        for (int it = 0; it <= T + 1; ++it) {
            if (it + 1 <= T) {
                publish((it + 1) & 1);
                if (it + 2 <= T) fetch(it + 2);
            }
            lds_barrier();
        }
    }
}

// ------------------------------------------------------------------------------------------ launchers
namespace {

template <int H, int P>
hipError_t act_dispatch(const NetFrags &net, int rows, const int32_t *env_index, int n_envs, const float *obs,
                        const uint8_t *avail, const float *h_in,
                        const uint8_t *reset, const int32_t *step_t, float epsilon, uint64_t seed, float *h_out,
                        int32_t *action, float *q_out, hipStream_t stream)
{
    constexpr int RPW = 32 * front_col_blocks(H, P) * kFrontWaves;     // rows per workgroup
    FrontArgs a{};
    a.net[0] = net;
    a.rows = rows; a.env_index = env_index; a.n_envs = n_envs; a.obs = obs; a.avail = avail; a.h_in = h_in; a.reset = reset; a.step_t = step_t;
    a.epsilon = epsilon; a.seed = seed; a.h_out = h_out; a.action = action; a.q_out = q_out; a.nets = 1;
    const dim3 grid((unsigned)((rows + RPW - 1) / RPW)), block(kFrontThreads);
    if (net.mb2 == 1) hipLaunchKernelGGL((front_kernel<H, P, 1, true>), grid, block, 0, stream, a);
    else              hipLaunchKernelGGL((front_kernel<H, P, 2, true>), grid, block, 0, stream, a);
    return hipGetLastError();
}

template <int H, int P>
hipError_t unroll_dispatch(const NetFrags &online, const NetFrags &target, bool two_nets, char *gi_on, char *gi_tg,
                           int B, int T, const int32_t *episode_index, int pool_episodes, const float *obs, const uint8_t *avail, const int32_t *actions,
                           const float *reward, const uint8_t *terminated, const uint8_t *filled, float gamma,
                           float *q_taken, float *next_max, float *td_target, float *q_all, hipStream_t stream,
                           hipEvent_t between, TdMode mode, int32_t *next_action)
{
    const int rows = B * online.N, tiles = (rows + 31) / 32;
    const unsigned nets = two_nets ? 2u : 1u;
    {
        constexpr int NC = front_col_blocks(H, P);
        const long groups = (long)((tiles + NC - 1) / NC) * (T + 1);      // wavefront work items
        FrontArgs a{};
        a.net[0] = online; a.net[1] = target;
        a.gi[0] = gi_on; a.gi[1] = gi_tg;
        a.B = B; a.T = T; a.episode_index = episode_index; a.pool_episodes = pool_episodes; a.obs = obs; a.nets = nets;
        const dim3 grid((unsigned)((groups + kFrontWaves - 1) / kFrontWaves) * nets), block(kFrontThreads);
        // the fc2 block count does not enter the projection; one instantiation serves both
        hipLaunchKernelGGL((front_kernel<H, P, 1, false>), grid, block, 0, stream, a);
        hipError_t err = hipGetLastError();
        if (err != hipSuccess) return err;
        if (between) {
            err = hipEventRecord(between, stream);
            if (err != hipSuccess) return err;
        }
    }
    const dim3 grid((unsigned)tiles, nets), block(64 * RecurrentShape<H, P>::kWaves);
    const int two = two_nets ? 1 : 0;
#define MARL_REC(MB, QA)                                                                                             \
    hipLaunchKernelGGL((recurrent_td_kernel<H, P, MB, QA>), grid, block, 0, stream, online, target, gi_on, gi_tg, two,  \
                       B, T, episode_index, pool_episodes, avail, actions, reward, terminated, filled, gamma, q_taken,      \
                       next_max, td_target, q_all, (int)mode, next_action)
    if (online.mb2 == 1) { if (q_all) MARL_REC(1, true); else MARL_REC(1, false); }
    else                 { if (q_all) MARL_REC(2, true); else MARL_REC(2, false); }
#undef MARL_REC
    return hipGetLastError();
}

}  // namespace

hipError_t launch_act_step(const NetFrags &net, int E, const int32_t *env_index, int n_listed, const float *obs,
                           const uint8_t *avail, const float *h_in,
                           const uint8_t *reset, const int32_t *step_t, float epsilon, uint64_t seed, float *h_out,
                           int32_t *action, float *q_out, hipStream_t stream)
{
    const int rows = (env_index ? n_listed : E) * net.N;
#define MARL_ACT(HH, PP) \
    return act_dispatch<HH, PP>(net, rows, env_index, E, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action, q_out, stream)
    if (net.H == 64 && net.planes == 2) MARL_ACT(64, 2);
    if (net.H == 64 && net.planes == 1) MARL_ACT(64, 1);
    if (net.H == 128 && net.planes == 2) MARL_ACT(128, 2);
    if (net.H == 128 && net.planes == 1) MARL_ACT(128, 1);
#undef MARL_ACT
    return hipErrorInvalidValue;
}

size_t unroll_scratch_bytes(const NetFrags &net, int B, int T)
{
    const size_t tiles = ((size_t)B * net.N + 31) / 32;
    const size_t block_bytes = net.planes == 1 ? GiLayout<1>::kBlockBytes : GiLayout<2>::kBlockBytes;
    return tiles * (size_t)(T + 1) * 3 * (net.H / 32) * block_bytes;
}

hipError_t launch_unroll_td(const NetFrags &online, const NetFrags &target, bool two_nets, void *scratch_online,
                            void *scratch_target, int B, int T, const int32_t *episode_index, int pool_episodes,
                            const float *obs, const uint8_t *avail,
                            const int32_t *actions, const float *reward, const uint8_t *terminated,
                            const uint8_t *filled, float gamma, float *q_taken, float *next_max, float *td_target,
                            float *q_all, hipStream_t stream, hipEvent_t between, TdMode mode, int32_t *next_action)
{
    if (mode != kTdPlain && (two_nets || !next_action)) return hipErrorInvalidValue;
    char *gi_on = static_cast<char *>(scratch_online), *gi_tg = static_cast<char *>(scratch_target);
#define MARL_UNROLL(HH, PP)                                                                                        \
    return unroll_dispatch<HH, PP>(online, target, two_nets, gi_on, gi_tg, B, T, episode_index, pool_episodes, obs, \
                                   avail, actions, reward,                                                         \
                                   terminated, filled, gamma, q_taken, next_max, td_target, q_all, stream, between,  \
                                   mode, next_action)
    if (online.H == 64 && online.planes == 2) MARL_UNROLL(64, 2);
    if (online.H == 64 && online.planes == 1) MARL_UNROLL(64, 1);
    if (online.H == 128 && online.planes == 2) MARL_UNROLL(128, 2);
    if (online.H == 128 && online.planes == 1) MARL_UNROLL(128, 1);
#undef MARL_UNROLL
    return hipErrorInvalidValue;
}

}  // namespace marl
