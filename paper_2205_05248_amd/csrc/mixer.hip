// Mixing network of the learner step (include/marl_mixer.h): handle, packing, kernel, entry points.
//
// The work is one dense contraction, [ (N + 3) M generated quantities x S ] . [ S x B T states ],
// followed by a cheap per-transition combination, done for the online mixer on state[b, t] and for
// the target mixer on state[b, t + 1].  A workgroup takes one of the two passes for 64 consecutive
// transitions (128 on large batches), one tile of 16 per wave; a wave keeps its tile's states in
// registers as MFMA B operands (bf16, plus the bf16 remainder for fp32 parameters) for the whole
// pass.  The state matrices stream past as A-operand fragments, one block of 16 generated quantities
// at a time: the block's fragments are copied global -> registers -> LDS by all waves while earlier
// blocks are being multiplied (asked for five blocks ahead), so every wave reads them from LDS and
// L2 sees each block once per workgroup.  A block's 16 x 16 result lands with lane (row c, quarter q)
// holding quantities 4 q .. 4 q + 3 of row c, and is folded into the running mix:
//   blocks of agent n        hidden += q[n] |result + hb1|
//   blocks of b1             hidden += result + hbb1
//   blocks of w2             total  += |result + hb2| elu(hidden)     (hidden is complete by then)
//   blocks of the offset     total  += v2 relu(result + c1)
// and at the end the row's four lanes add their totals.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "../../include/marl_mixer.h"
#include "fused16.h"
#include "qnet_internal.h"

struct marl_mixer {
    marl_mixer_desc desc;
    int planes;                  // 1: bf16 matrices, 2: bf16 + remainder
    int ks;                      // k-steps of 32 over the state
    void *image;                 // device: fragments, then the fp32 tables
    const marl::bf16x8 *frags;   // [(N + 3) M / 16][ks][planes][64]
    const float *bias;           // [(N + 3) M]: hb1 | hbb1 | hb2 | c1
    const float *v2;             // [M]
    const float *c2;             // [1]
    size_t bytes;                // of the image
    void *staging;               // pinned host copy of the image for marl_mixer_set_weights (lazily allocated)
    hipEvent_t staging_done;     // the last upload from it
    // device-side refresh (marl_mixer_sgd_step), built on first use: source parameter of every 16-bit element
    // of the fragments, then of every fp32 table entry
    int32_t *repack_map;
    size_t frag_elems, table_entries;
};

namespace marl {
namespace {

constexpr int kBigTiles = 1, kBigWaves = 8;       // shape of a workgroup on large batches: tiles per wave, waves
constexpr int kAhead = 4;             // blocks between asking for a block's fragments and multiplying them

struct MixerArgs {
    const bf16x8 *frags[2];
    const float *bias[2], *v2[2];
    const float *c2[2];
    int N, S, ks, rows, T;                 // ks: padded k-steps of the packed fragments
    const float *state, *q[2], *reward;
    const uint8_t *terminated, *filled;
    float gamma;
    float *q_total, *y_total, *td_err;
};

// The larger workgroup shape needs two register sets of a block's fragments, and pays off once the
// state is long enough for the fragment traffic to matter.
template <int P, int KS> constexpr bool mixer_big_shape_fits() { return KS * P <= 16 && KS >= 8; }

// Streams blocks of 16 generated quantities past the waves of a workgroup: fragments travel
// global -> registers -> LDS, and every wave multiplies each block with its own tiles' states.  A
// block is asked for kAhead (+ 1) blocks before it is multiplied (an L2 round trip is several blocks
// long) into one of kAhead register sets, indexed by block % kAhead with the loop unrolled over them
// so that a wait covers only that set.  Blocks past the last one re-read it (their results are the
// caller's to ignore), which keeps every step the same straight-line code with no other global load
// in it: biases and agent values come from LDS.
template <int P, int KS, int W>
struct BlockStream {
    static constexpr int kThreads = 64 * W;
    static constexpr int kChunk = KS * P * 64;                             // 16-byte vectors of one block
    static constexpr int kStage = (kChunk + kThreads - 1) / kThreads;      // vectors per thread and block
    static constexpr bool kReadAhead = KS * P <= 16;                       // two register sets of a block's fragments fit
    static constexpr size_t kLdsBytes = (size_t)2 * kChunk * 16;           // two block buffers
    const bf16x8 *frags;
    int n_blocks;
    bf16x8 *buf;
    bf16x8 stage[kAhead][kStage];

    __device__ __forceinline__ void fetch_one(int set, int blk, int i)
    {
        const bf16x8 *src = frags + (size_t)min(blk, n_blocks - 1) * kChunk;
        stage[set][i] = src[min(i * kThreads + (int)threadIdx.x, kChunk - 1)];
    }
    __device__ __forceinline__ void fetch(int set, int blk)
    {
#pragma unroll
        for (int i = 0; i < kStage; ++i) fetch_one(set, blk, i);
    }
    __device__ __forceinline__ void stash_one(int set, int blk, int i)
    {
        const int at = i * kThreads + threadIdx.x;
        if (kChunk % kThreads == 0 || at < kChunk) buf[(size_t)(blk & 1) * kChunk + at] = stage[set][i];
    }
    __device__ __forceinline__ void stash(int set, int blk)
    {
#pragma unroll
        for (int i = 0; i < kStage; ++i) stash_one(set, blk, i);
    }
    // asks for the first blocks; nothing of LDS is touched yet
    __device__ __forceinline__ void begin(const bf16x8 *blocks, int count, bf16x8 *lds_buffers)
    {
        frags = blocks;
        n_blocks = count;
        buf = lds_buffers;
#pragma unroll
        for (int u = 0; u < kAhead; ++u) fetch(u, u);
    }
    // Multiplies every block with the wave's TPW tiles and hands the 16 x 16 results to
    // fold(tile, blk % MB, blk, result, agent value).  bias: the streamed blocks' bias table in LDS;
    // qv: the wave's agent values in LDS, [tile][agent][row], n_q agents (block blk belongs to agent
    // blk / MB; later blocks get the last agent's value, to ignore).  The workgroup must have
    // finished with the block buffers and written bias and qv before the call (the first barrier
    // inside orders the latter).
    template <int MB, int TPW, typename Fold>
    __device__ __forceinline__ void run(const Frag<P> (&st)[TPW][KS], const float *bias, const float *qv, int n_q, Fold &&fold)
    {
        static_assert(kAhead % MB == 0, "a block's place among its group's blocks follows from the step number");
        const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
        if constexpr (kReadAhead) {
            // One wave issues in order, so whatever is to run beside the products has to sit between
            // them in the instruction stream.  A step multiplies block b from one register set while,
            // k-step by k-step, block b + 1 is read from LDS into the other set (by the block's
            // parity), the step's share of block b + 5 is asked for and block b + 2 is written to
            // LDS: its buffer held block b, whose reads every wave finished before the barrier that
            // ended the previous step.  Bias and agent value of block b + 1 are read at the head of
            // the step.
            static_assert(2 * kStage <= KS, "a step's loads and its LDS writes sit at different k-steps");
            WFrag<P> w[2][KS];
            auto read_step = [&](int set, int blk, int ks) {
                const bf16x8 *src = buf + (size_t)(blk & 1) * kChunk + lane;
                w[set][ks].hi = src[(ks * P) * 64];
                if constexpr (P == 2) w[set][ks].lo = src[(ks * P + 1) * 64];
            };
            auto head = [&](int blk, f32x4 &bias4, float (&qn)[TPW]) {
                bias4 = load_feature4(bias, min(blk, n_blocks - 1), q4);
#pragma unroll
                for (int i = 0; i < TPW; ++i) qn[i] = qv[(i * n_q + min(blk / MB, n_q - 1)) * 16 + c];
            };
            stash(0, 0);
            stash(1, 1);
            fetch(0, kAhead);
            lds_barrier();
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) read_step(0, 0, ks);
            f32x4 bias_next;
            float qn_next[TPW];
            head(0, bias_next, qn_next);
            lds_barrier();                         // every wave holds block 0 before its buffer is written again
            for (int base = 0; base < n_blocks; base += kAhead) {
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int blk = base + u;
                    f32x4 acc[TPW];
                    float qn[TPW];
#pragma unroll
                    for (int i = 0; i < TPW; ++i) {
                        acc[i] = bias_next;
                        qn[i] = qn_next[i];
                    }
                    head(blk + 1, bias_next, qn_next);
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                        for (int i = 0; i < TPW; ++i) mma16<P>(acc[i], w[u & 1][ks], st[i][ks]);
                        read_step((u + 1) & 1, blk + 1, ks);
                        if (ks < kStage) fetch_one((u + 1) % kAhead, blk + kAhead + 1, ks);      // that set held block blk + 1, in LDS since the last step
                        if (ks >= KS - kStage) stash_one((u + 2) % kAhead, blk + 2, ks - (KS - kStage));
                        __builtin_amdgcn_sched_barrier(0);
                    }
#pragma unroll
                    for (int i = 0; i < TPW; ++i) fold(i, u % MB, blk, acc[i], qn[i]);
                    lds_barrier();
                }
            }
        } else {
            static_assert(TPW == 1, "more tiles per wave come with the read-ahead loop");
            stash(0, 0);
            lds_barrier();
            for (int base = 0; base < n_blocks; base += kAhead) {
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int blk = base + u;
                    fetch(u, blk + kAhead);                            // this set held block blk, already in LDS
                    const bf16x8 *src = buf + (size_t)(blk & 1) * kChunk + lane;
                    WFrag<P> w[KS];
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) {
                        w[ks].hi = src[(ks * P) * 64];
                        if constexpr (P == 2) w[ks].lo = src[(ks * P + 1) * 64];
                    }
                    f32x4 acc = load_feature4(bias, min(blk, n_blocks - 1), q4);
                    const float qn = qv[min(blk / MB, n_q - 1) * 16 + c];
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks) mma16<P>(acc, w[ks], st[0][ks]);
                    fold(0, u % MB, blk, acc, qn);
                    stash((u + 1) % kAhead, blk + 1);
                    lds_barrier();
                }
            }
        }
    }
};

// What a wave needs of its tiles before the blocks stream: the bias table and the tiles' agent values in
// LDS, the tiles' states as B operands in registers; `stream.begin` is called once every load of the
// prologue has been issued.  Everything is asked for before any of it is used, smallest first (loads
// answer in order): a loop of load-then-store over a run-time count would pay a memory round trip per
// iteration.  slot_shift: 0 the slot's own state, 1 the next slot's.
template <int P, int KS, int TPW, int W>
__device__ __forceinline__ void mixer_prologue(const float *bias_src, int F, float *bias_lds, const float *q_src, int N, float *q_lds,
                                               const float *state, int S, int T, int rows, int slot_shift, int (&row)[TPW],
                                               Frag<P> (&st)[TPW][KS], BlockStream<P, KS, W> &stream, const bf16x8 *blocks, int n_blocks,
                                               bf16x8 *buf)
{
    constexpr int kThreads = 64 * W, kBatch = 8;
    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    {
        const f32x4 *src = reinterpret_cast<const f32x4 *>(bias_src);          // F is a multiple of 16, the table 16-byte aligned
        f32x4 *dst = reinterpret_cast<f32x4 *>(bias_lds);
        for (int i0 = threadIdx.x; i0 < F / 4; i0 += 4 * kThreads) {
            f32x4 v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = src[min(i0 + e * kThreads, F / 4 - 1)];
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (i0 + e * kThreads < F / 4) dst[i0 + e * kThreads] = v[e];
        }
    }
    // The tiles' states as B operands: lane (row c, quarter q) holds values 32 ks + 8 q + 0..7.
    // K-steps wholly inside the row are two 16-byte loads (only 4-byte alignment is assumed); a
    // partial one is read element by element from positions clamped into the row and zeroed past
    // its end.  Rows past the end re-read the last one.
    const int nfull = S / 32;
    const float *srow[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int tile_row0 = ((blockIdx.x * W + wave) * TPW + i) * 16;
        row[i] = tile_row0 + c;
        const int rr = min(row[i], rows - 1);
        srow[i] = state + ((size_t)(rr / T) * (T + 1) + rr % T + slot_shift) * S;
        for (int k0 = lane; k0 < 16 * N; k0 += 64 * kBatch) {      // the tile's agent values: its rows are consecutive in memory
            float v[kBatch];
#pragma unroll
            for (int e = 0; e < kBatch; ++e) {
                const int k = min(k0 + 64 * e, 16 * N - 1);
                v[e] = q_src[(size_t)min(tile_row0 + k / N, rows - 1) * N + k % N];
            }
#pragma unroll
            for (int e = 0; e < kBatch; ++e) {
                const int k = k0 + 64 * e;
                if (k < 16 * N) q_lds[(i * N + k % N) * 16 + k / N] = v[e];
            }
        }
    }
    if (nfull == KS) {                         // the state fills its k-steps: every load first, then the first blocks' fragments
        f32x4 raw[TPW][KS][2];
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                __builtin_memcpy(&raw[i][ks][0], srow[i] + 32 * ks + 8 * q4, 16);
                __builtin_memcpy(&raw[i][ks][1], srow[i] + 32 * ks + 8 * q4 + 4, 16);
            }
        stream.begin(blocks, n_blocks, buf);
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 4; ++e) { v[e] = raw[i][ks][0][e]; v[4 + e] = raw[i][ks][1][e]; }
                st[i][ks] = to_frag<P>(v);
            }
    } else {
        stream.begin(blocks, n_blocks, buf);
#pragma unroll
        for (int i = 0; i < TPW; ++i)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                float v[8];
                if (ks < nfull) {
                    f32x4 lo4, hi4;
                    __builtin_memcpy(&lo4, srow[i] + 32 * ks + 8 * q4, 16);
                    __builtin_memcpy(&hi4, srow[i] + 32 * ks + 8 * q4 + 4, 16);
#pragma unroll
                    for (int e = 0; e < 4; ++e) { v[e] = lo4[e]; v[4 + e] = hi4[e]; }
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const int at = 32 * ks + 8 * q4 + e;
                        const float x = srow[i][min(at, S - 1)];
                        v[e] = at < S ? x : 0.0f;
                    }
                }
                st[i][ks] = to_frag<P>(v);
            }
    }
}

// One pass of one group of 16 W TPW transitions: blockIdx.y = 0 is the online mixer on the chosen
// values and the slot's state (Q_total), 1 the target mixer on the bootstrap values and the next
// slot's state (y_total).  td_err = filled ? y_total - Q_total : 0 is formed by both passes adding
// their term to an array cleared beforehand: the two orders give the same bits (0 + x = x, and
// -Q + y and y + (-Q) round alike).
// KS: k-steps of 32 over the state (the packed fragments are zero past the state's end).
// TPW: tiles of 16 transitions per wave; each fragment read from LDS then feeds TPW products.
// W: wavefronts per workgroup, one (4) or two (8) per SIMD.
template <int MB, int P, int KS, int TPW, int W>
__global__ __launch_bounds__(64 * W) void mixer_td_kernel(const MixerArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int lane = threadIdx.x & 63, q4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int pass = blockIdx.y;
    const int N = a.N;
    const int n_blocks = (N + 3) * MB, F = n_blocks * 16;
    using Stream = BlockStream<P, KS, W>;
    // LDS: two block buffers, the pass's bias table, the tiles' agent values [wave][tile][agent][row]
    bf16x8 *const buf = reinterpret_cast<bf16x8 *>(lds);
    float *const bias_lds = reinterpret_cast<float *>(lds + Stream::kLdsBytes);
    float *const q_lds = bias_lds + F + (size_t)wave * TPW * N * 16;

    Stream stream;
    const float c2 = a.c2[pass][0];
    Frag<P> st[TPW][KS];
    int row[TPW];
    mixer_prologue<P, KS, TPW, W>(a.bias[pass], F, bias_lds, a.q[pass], N, q_lds, a.state, a.S, a.T, a.rows, pass, row, st, stream,
                                  a.frags[pass], n_blocks, buf);
    f32x4 gain[MB];                            // v2, this lane's units
#pragma unroll
    for (int j = 0; j < MB; ++j) gain[j] = load_feature4(a.v2[pass], j, q4);
    // what the end of the pass reads, asked for now
    float reward[TPW];
    bool live[TPW], open_end[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int rr = min(row[i], a.rows - 1);
        reward[i] = a.reward[rr];
        live[i] = a.filled[rr] != 0;
        open_end[i] = a.terminated[rr] == 0;
    }
    f32x4 hidden[TPW][MB];
    float total[TPW];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        total[i] = 0.0f;
#pragma unroll
        for (int j = 0; j < MB; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) hidden[i][j][r] = 0.0f;
    }
    // A block's 16 x 16 result of tile i, folded into the tile's running mix.  Agent and b1 blocks take
    // the same straight-line code with two coefficients (q[n], 0) or (0, 1): a product with zero adds
    // nothing and a product with one is exact, so the sums are the ones of `hidden += q[n] |result|`
    // and `hidden += result`.  Only the last blocks branch (uniformly, around arithmetic alone).
    auto fold = [&](int i, int j, int blk, const f32x4 &acc, float qn) {
        const int group = blk / MB;                                // agents 0 .. N-1, then b1, w2, offset
        const float by_abs = group < N ? qn : 0.0f, by_value = group == N ? 1.0f : 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) hidden[i][j][r] = fmaf(by_value, acc[r], fmaf(by_abs, fabsf(acc[r]), hidden[i][j][r]));
        if (group == N + 1) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float x = hidden[i][j][r];
                total[i] = fmaf(fabsf(acc[r]), x > 0.0f ? x : expm1f(x), total[i]);
            }
        } else if (group == N + 2) {
#pragma unroll
            for (int r = 0; r < 4; ++r) total[i] = fmaf(gain[j][r], fmaxf(acc[r], 0.0f), total[i]);
        }
    };
    stream.template run<MB, TPW>(st, bias_lds, q_lds, N, fold);
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        float sum = total[i];
        sum += __shfl_xor(sum, 16);
        sum += __shfl_xor(sum, 32);
        const float mixed = sum + c2;
        const int r = row[i];
        if (r < a.rows && q4 == 0) {
            if (pass == 0) {
                if (a.q_total) a.q_total[r] = mixed;
                if (a.td_err && live[i]) atomicAdd(a.td_err + r, -mixed);
            } else {
                const float y = reward[i] + a.gamma * (open_end[i] ? 1.0f : 0.0f) * mixed;
                if (a.y_total) a.y_total[r] = y;
                if (a.td_err && live[i]) atomicAdd(a.td_err + r, y);
            }
        }
    }
}

__global__ __launch_bounds__(256) void mixer_clear_kernel(float *__restrict__ x, int n)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < n) x[i] = 0.0f;
}

// loss[0] = sum of the squared errors, loss[1] = number of filled transitions.  One workgroup, each
// thread a strided partial sum, then a tree over LDS: the summation order is fixed, so the result is
// the same on every run.
__global__ __launch_bounds__(256) void mixer_loss_kernel(const float *__restrict__ td_err, const uint8_t *__restrict__ filled,
                                                        int rows, float *__restrict__ loss)
{
    __shared__ float sq[256], cnt[256];
    float s = 0.0f, n = 0.0f;
    // eight loads in flight per thread (positions past the end clamped, their terms dropped); the terms are
    // added in the same order as one by one
    for (int i0 = threadIdx.x; i0 < rows; i0 += 256 * 8) {
        float e[8];
        uint8_t f[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const int i = min(i0 + 256 * k, rows - 1);
            e[k] = td_err[i];
            f[k] = filled[i];
        }
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (i0 + 256 * k < rows) {
                s = fmaf(e[k], e[k], s);
                n += f[k] ? 1.0f : 0.0f;
            }
    }
    sq[threadIdx.x] = s;
    cnt[threadIdx.x] = n;
    __syncthreads();
    for (int half = 128; half >= 1; half >>= 1) {
        if ((int)threadIdx.x < half) {
            sq[threadIdx.x] += sq[threadIdx.x + half];
            cnt[threadIdx.x] += cnt[threadIdx.x + half];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        loss[0] = sq[0];
        loss[1] = cnt[0];
    }
}

template <int MB, int P, int KS, int TPW, int W>
hipError_t mixer_launch_shape(const MixerArgs &a, hipStream_t stream)
{
    const int per_group = 16 * W * TPW;
    const dim3 grid((unsigned)((a.rows + per_group - 1) / per_group), 2), block(64 * W);
    const size_t lds = (size_t)2 * KS * P * 1024 + sizeof(float) * ((size_t)(a.N + 3) * MB * 16 + (size_t)W * TPW * a.N * 16);
    hipError_t err = allow_large_lds<mixer_td_kernel<MB, P, KS, TPW, W>>(kLdsLimit);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((mixer_td_kernel<MB, P, KS, TPW, W>), grid, block, lds, stream, a);
    return hipGetLastError();
}

// Once groups of 64 transitions would give more workgroups than there are compute units, a workgroup
// takes 128 with eight waves: a block's fragments then come from L2 half as often, and with two waves
// on a SIMD one's LDS reads (a wave issues a 16-byte-per-lane read only every ~29 cycles) run beside
// the other's products.
template <int MB, int P, int KS>
hipError_t mixer_launch(const MixerArgs &a, hipStream_t stream)
{
    if constexpr (mixer_big_shape_fits<P, KS>()) {
        int dev = 0, n_cu = 0;
        if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            n_cu = 256;
        if (2 * ((a.rows + 63) / 64) > n_cu) return mixer_launch_shape<MB, P, KS, kBigTiles, kBigWaves>(a, stream);
    }
    return mixer_launch_shape<MB, P, KS, 1, 4>(a, stream);
}

template <int P, int KS>
hipError_t mixer_dispatch(int mb, const MixerArgs &a, hipStream_t stream)
{
    switch (mb) {
    case 1: return mixer_launch<1, P, KS>(a, stream);
    case 2: return mixer_launch<2, P, KS>(a, stream);
    case 4: return mixer_launch<4, P, KS>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

// The kernels exist for these numbers of k-steps; a state is padded (with zero fragments) to the next.
constexpr int kStepChoices[] = {2, 4, 6, 8, 16, 32};
int padded_ksteps(int S)
{
    const int ks = (S + 31) / 32;
    for (int choice : kStepChoices)
        if (ks <= choice) return choice;
    return 0;
}

template <int P>
hipError_t mixer_dispatch_ks(int ks, int mb, const MixerArgs &a, hipStream_t stream)
{
    switch (ks) {
    case 2: return mixer_dispatch<P, 2>(mb, a, stream);
    case 4: return mixer_dispatch<P, 4>(mb, a, stream);
    case 6: return mixer_dispatch<P, 6>(mb, a, stream);
    case 8: return mixer_dispatch<P, 8>(mb, a, stream);
    case 16: return mixer_dispatch<P, 16>(mb, a, stream);
    case 32: if constexpr (P == 1) return mixer_dispatch<1, 32>(mb, a, stream);
    default: return hipErrorInvalidValue;
    }
}

bool mixer_desc_valid(const marl_mixer_desc *d, int *why)
{
    if (d->weight_dtype != MARL_DTYPE_F32 && d->weight_dtype != MARL_DTYPE_BF16) {
        *why = MARL_ERR_BAD_DTYPE;
        return false;
    }
    const int s_max = d->weight_dtype == MARL_DTYPE_BF16 ? MARL_MIXER_MAX_STATE_BF16 : MARL_MIXER_MAX_STATE_F32;
    if (d->n_agents < 1 || d->n_agents > MARL_MAX_AGENTS || (d->embed != 16 && d->embed != 32 && d->embed != 64) ||
        d->state_dim < 1 || d->state_dim > s_max || d->device < 0) {
        *why = MARL_ERR_BAD_DIM;
        return false;
    }
    return true;
}

size_t mixer_params(const marl_mixer_desc *d)
{
    const size_t N = d->n_agents, M = d->embed, S = d->state_dim;
    return (N * M + 3 * M) * (S + 1) + M + 1;
}

struct MixerDeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit MixerDeviceGuard(int dev) { ok = hipGetDevice(&prev) == hipSuccess && hipSetDevice(dev) == hipSuccess; }
    ~MixerDeviceGuard() { if (ok && prev >= 0) (void)hipSetDevice(prev); }
};

}  // namespace
}  // namespace marl

extern "C" {

size_t marl_mixer_param_count(const marl_mixer_desc *desc)
{
    int why;
    if (!desc || !marl::mixer_desc_valid(desc, &why)) return 0;
    return marl::mixer_params(desc);
}

}  // extern "C"

namespace marl {
namespace {
// The device image of a mixer: fragments of the four state matrices in the order the kernel walks
// them (W1 rows agent-major, b1, w2, offset layer), then the fp32 tables hb1 | hbb1 | hb2 | c1, v2, c2.
// Returns a calloc'ed host copy (caller frees) or null.
char *pack_mixer_image(const marl_mixer_desc &d, const float *w, size_t *bytes, size_t *frag_bytes)
{
    const int N = d.n_agents, M = d.embed, S = d.state_dim;
    const int planes = d.weight_dtype == MARL_DTYPE_BF16 ? 1 : 2;
    const int ks = padded_ksteps(S), F = (N + 3) * M;
    const float *Hw1 = w, *hb1 = Hw1 + (size_t)N * M * S, *Hb1 = hb1 + (size_t)N * M, *hbb1 = Hb1 + (size_t)M * S;
    const float *Hw2 = hbb1 + M, *hb2 = Hw2 + (size_t)M * S, *V1 = hb2 + M, *c1 = V1 + (size_t)M * S, *v2 = c1 + M, *c2 = v2 + M;
    *frag_bytes = (size_t)(F / 16) * ks * planes * 1024;
    *bytes = *frag_bytes + sizeof(float) * (F + M + 4);
    char *host = static_cast<char *>(std::calloc(1, *bytes));
    if (!host) return nullptr;
    uint16_t *frags = reinterpret_cast<uint16_t *>(host);
    const size_t per_block = (size_t)ks * planes * 512;
    auto pack_rows = [&](int first_block, const float *W, int n_rows) {      // blocks of 16 rows, ks k-steps each (zero past S)
        for (int fb = 0; fb < n_rows / 16; ++fb)
            pack_frags16(frags + (size_t)(first_block + fb) * per_block, W + (size_t)16 * fb * S, 16, S, S, false, planes);
    };
    pack_rows(0, Hw1, N * M);
    pack_rows(N * M / 16, Hb1, M);
    pack_rows((N + 1) * M / 16, Hw2, M);
    pack_rows((N + 2) * M / 16, V1, M);
    float *bias = reinterpret_cast<float *>(host + *frag_bytes);
    std::memcpy(bias, hb1, sizeof(float) * N * M);
    std::memcpy(bias + (size_t)N * M, hbb1, sizeof(float) * M);
    std::memcpy(bias + (size_t)(N + 1) * M, hb2, sizeof(float) * M);
    std::memcpy(bias + (size_t)(N + 2) * M, c1, sizeof(float) * M);
    std::memcpy(bias + F, v2, sizeof(float) * M);
    bias[F + M] = c2[0];
    return host;
}
}  // namespace
}  // namespace marl

extern "C" {

int marl_mixer_create(const marl_mixer_desc *desc, const float *host_weights, size_t n_weights, marl_mixer **out)
{
    if (!desc || !host_weights || !out) return MARL_ERR_NULL;
    *out = nullptr;
    int why;
    if (!marl::mixer_desc_valid(desc, &why)) return why;
    if (n_weights != marl::mixer_params(desc)) return MARL_ERR_MISMATCH;
    size_t bytes, frag_bytes;
    char *host = marl::pack_mixer_image(*desc, host_weights, &bytes, &frag_bytes);
    if (!host) return MARL_ERR_NOMEM;
    marl_mixer *m = new (std::nothrow) marl_mixer();
    if (!m) { std::free(host); return MARL_ERR_NOMEM; }
    const int F = (desc->n_agents + 3) * desc->embed;
    m->desc = *desc;
    m->planes = desc->weight_dtype == MARL_DTYPE_BF16 ? 1 : 2;
    m->ks = marl::padded_ksteps(desc->state_dim);
    m->image = nullptr; m->bytes = bytes; m->staging = nullptr; m->staging_done = nullptr;
    m->repack_map = nullptr; m->frag_elems = 0; m->table_entries = 0;
    marl::MixerDeviceGuard guard(desc->device);
    hipError_t err = guard.ok ? hipMalloc(&m->image, bytes) : hipErrorInvalidDevice;
    if (err == hipSuccess) err = hipMemcpy(m->image, host, bytes, hipMemcpyHostToDevice);
    std::free(host);
    if (err != hipSuccess) {
        if (m->image) (void)hipFree(m->image);
        delete m;
        return err == hipErrorOutOfMemory ? MARL_ERR_NOMEM : marl::report_device_error(err, "marl_mixer_create");
    }
    m->frags = static_cast<const marl::bf16x8 *>(m->image);
    m->bias = reinterpret_cast<const float *>(static_cast<char *>(m->image) + frag_bytes);
    m->v2 = m->bias + F;
    m->c2 = m->v2 + desc->embed;
    *out = m;
    return MARL_OK;
}

int marl_mixer_set_weights(marl_mixer *m, const float *host_weights, size_t n_weights, void *hip_stream)
{
    if (!m || !host_weights) return MARL_ERR_NULL;
    if (n_weights != marl::mixer_params(&m->desc)) return MARL_ERR_MISMATCH;
    size_t bytes, frag_bytes;
    char *host = marl::pack_mixer_image(m->desc, host_weights, &bytes, &frag_bytes);
    if (!host) return MARL_ERR_NOMEM;
    struct FreeHost { void *p; ~FreeHost() { std::free(p); } } free_host{host};
    marl::MixerDeviceGuard guard(m->desc.device);
    if (!guard.ok) return marl::report_device_error(hipErrorInvalidDevice, "hipSetDevice");
    hipError_t err;
    if (!m->staging) {
        err = hipHostMalloc(&m->staging, bytes, hipHostMallocDefault);
        if (err != hipSuccess) { m->staging = nullptr; return err == hipErrorOutOfMemory ? MARL_ERR_NOMEM : marl::report_device_error(err, "hipHostMalloc"); }
        err = hipEventCreateWithFlags(&m->staging_done, hipEventDisableTiming);
        if (err != hipSuccess) { (void)hipHostFree(m->staging); m->staging = nullptr; m->staging_done = nullptr; return marl::report_device_error(err, "hipEventCreate"); }
    } else {
        err = hipEventSynchronize(m->staging_done);                      // the previous upload still reads the buffer
        if (err != hipSuccess) return marl::report_device_error(err, "hipEventSynchronize");
    }
    std::memcpy(m->staging, host, bytes);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    err = hipMemcpyAsync(m->image, m->staging, bytes, hipMemcpyHostToDevice, stream);
    if (err == hipSuccess) err = hipEventRecord(m->staging_done, stream);
    if (err != hipSuccess) return marl::report_device_error(err, "marl_mixer_set_weights");
    return MARL_OK;
}

void marl_mixer_destroy(marl_mixer *m)
{
    if (!m) return;
    marl::MixerDeviceGuard guard(m->desc.device);
    if (m->image) (void)hipFree(m->image);              // synchronises the device
    if (m->repack_map) (void)hipFree(m->repack_map);
    if (m->staging) (void)hipHostFree(m->staging);
    if (m->staging_done) (void)hipEventDestroy(m->staging_done);
    delete m;
}

int marl_mixer_td(marl_mixer *online, marl_mixer *target, int32_t B, int32_t T, const float *state,
                  const float *q_taken, const float *next_max, const float *reward, const uint8_t *terminated,
                  const uint8_t *filled, float gamma, float *q_total, float *y_total, float *td_err, float *loss,
                  void *hip_stream)
{
    if (!online) return MARL_ERR_NULL;
    if (loss && !td_err) return MARL_ERR_NULL;             // the loss is reduced from td_err
    if (!target) target = online;
    if (std::memcmp(&online->desc, &target->desc, sizeof(marl_mixer_desc)) != 0) return MARL_ERR_MISMATCH;
    if (B < 0 || T < 1 || (int64_t)B * T >= (int64_t)1 << 30) return MARL_ERR_BAD_DIM;
    if (!(std::isfinite(gamma) && gamma >= 0.0f && gamma <= 1.0f)) return MARL_ERR_BAD_ARG;
    if (B == 0) return MARL_OK;
    if (!state || !q_taken || !next_max || !reward || !terminated || !filled) return MARL_ERR_NULL;
    marl::MixerDeviceGuard guard(online->desc.device);
    if (!guard.ok) return marl::report_device_error(hipErrorInvalidDevice, "hipSetDevice");
    marl::MixerArgs a{};
    a.frags[0] = online->frags; a.frags[1] = target->frags;
    a.bias[0] = online->bias; a.bias[1] = target->bias;
    a.v2[0] = online->v2; a.v2[1] = target->v2;
    a.c2[0] = online->c2; a.c2[1] = target->c2;
    a.N = online->desc.n_agents; a.S = online->desc.state_dim; a.ks = online->ks; a.rows = B * T; a.T = T;
    a.state = state; a.q[0] = q_taken; a.q[1] = next_max; a.reward = reward; a.terminated = terminated; a.filled = filled;
    a.gamma = gamma; a.q_total = q_total; a.y_total = y_total; a.td_err = td_err;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int mb = online->desc.embed / 16;
    hipError_t err;
    if (td_err) {                                          // both passes add their term to it
        hipLaunchKernelGGL(marl::mixer_clear_kernel, dim3((unsigned)((a.rows + 255) / 256)), dim3(256), 0, stream, td_err, a.rows);
        err = hipGetLastError();
        if (err != hipSuccess) return marl::report_device_error(err, "marl_mixer_td clear launch");
    }
    if (online->planes == 2) err = marl::mixer_dispatch_ks<2>(a.ks, mb, a, stream);
    else err = marl::mixer_dispatch_ks<1>(a.ks, mb, a, stream);
    if (err != hipSuccess) return marl::report_device_error(err, "marl_mixer_td launch");
    if (loss) {
        hipLaunchKernelGGL(marl::mixer_loss_kernel, dim3(1), dim3(256), 0, stream, td_err, filled, a.rows, loss);
        err = hipGetLastError();
        if (err != hipSuccess) return marl::report_device_error(err, "marl_mixer_td loss launch");
    }
    return MARL_OK;
}

}  // extern "C"

// ------------------------------------------------------------------------------------------ backward pass
// Gradient of sum_i e[i] Q_total[i] (e = dL/dQ_total, the caller's) with respect to the mixer's parameters and
// to the agents' values.  Two stages:
//   mixer_back_kernel   a workgroup takes 16 transitions: all (N + 3) M generated quantities again (the same
//                       MFMA contraction as the forward pass, fragments read from L2, results to LDS), the
//                       mix, and then the adjoint of every generated quantity, written to the workspace as a
//                       matrix [transitions, (N + 3) M + M + 1] (the last M + 1 columns: e relu(offset unit), e),
//                       and dL/dq for the agents' networks;
//   launch_tn_product   every state matrix's gradient is (adjoint columns)^T [state | 1] summed over the
//                       transitions: the sample-contraction product of the Q-network's backward pass, cut into
//                       slices of rows and state columns that fit its two shapes.
namespace marl {
namespace {

struct MixerBackArgs {
    const bf16x8 *frags;
    const float *bias, *v2;
    int N, M, S, ks, rows, T, F, ldd;
    const float *state, *q, *e;
    void *dgen;         // [rows, ldd]: fp32, or bf16 for a one-plane mixer (whose products round the adjoints to bf16 anyway)
    float *grad_q;      // [rows, N]
};

// The adjoints are computed as the forward pass computes the mix: a workgroup of W waves takes 16 W
// transitions, the fragments stream past through LDS (BlockStream) and nothing but a tile's states, its
// hidden units and their adjoints is kept, in registers.  The blocks stream three times:
//   agents and b1         hidden pre-activation of every unit (as the forward pass)
//   w2 and offset         with the hidden units known: adjoints of the hidden pre-activations, of the w2 and
//                         offset quantities, and the columns for v2 and c2
//   agents again          each quantity once more, to give its adjoint (sign, agent value, adjoint of its
//                         unit) and its share of dL/dq
// so L2 serves every block three times per 16 W transitions instead of once per 16, and no generated
// quantity is stored.  Every store goes through a buffer descriptor, rows past the end and padding blocks
// at an offset the hardware drops, so the streaming steps stay straight-line code.
template <int MB, int P, int KS, int W>
__global__ __launch_bounds__(64 * W) void mixer_back_stream_kernel(const MixerBackArgs a)
{
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const int lane = threadIdx.x & 63, q4 = lane >> 4;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int N = a.N, M = a.M, F = a.F;
    using Stream = BlockStream<P, KS, W>;
    bf16x8 *const buf = reinterpret_cast<bf16x8 *>(lds);
    float *const bias_lds = reinterpret_cast<float *>(lds + Stream::kLdsBytes);
    float *const q_lds = bias_lds + F + (size_t)wave * N * 16;

    Stream stream;
    Frag<P> st[1][KS];
    int row[1];
    mixer_prologue<P, KS, 1, W>(a.bias, F, bias_lds, a.q, N, q_lds, a.state, a.S, a.T, a.rows, 0, row, st, stream, a.frags,
                                (N + 1) * MB, buf);
    const bool valid = row[0] < a.rows;
    const float e = a.e[min(row[0], a.rows - 1)];
    f32x4 gain[MB];                            // v2, this lane's units
#pragma unroll
    for (int j = 0; j < MB; ++j) gain[j] = load_feature4(a.v2, j, q4);
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr uint32_t kDrop = 0xFFFFFFF0u;
    constexpr uint32_t kElem = P == 1 ? 2u : 4u;                   // bytes per stored adjoint
    const __amdgpu_buffer_rsrc_t dgen_buf = __builtin_amdgcn_make_buffer_rsrc(a.dgen, 0, (int)((uint32_t)a.rows * (uint32_t)a.ldd * kElem), kRawBuffer);
    const __amdgpu_buffer_rsrc_t gq_buf = __builtin_amdgcn_make_buffer_rsrc(a.grad_q, 0, (int)((uint32_t)a.rows * (uint32_t)N * 4u), kRawBuffer);
    uint32_t drop = valid ? 0u : kDrop;
    asm volatile("" : "+v"(drop));
    const uint32_t row_at = (uint32_t)min(row[0], a.rows - 1) * (uint32_t)a.ldd;       // first element of the row in dgen
    auto store4 = [&](const f32x4 &v, uint32_t column, uint32_t drop_mask) {
        if constexpr (P == 1) {
            typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            bf16x4 r;
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = (__bf16)v[i];
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, r), dgen_buf, ((row_at + column) * 2u) | drop_mask, 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), dgen_buf, ((row_at + column) * 4u) | drop_mask, 0, 0);
        }
    };

    // 1. hidden pre-activations
    f32x4 hidden[MB];
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) hidden[j][r] = 0.0f;
    stream.template run<MB, 1>(st, bias_lds, q_lds, N, [&](int, int j, int blk, const f32x4 &acc, float qn) {
        const int group = blk / MB;
        const float by_abs = group < N ? qn : 0.0f, by_value = group == N ? 1.0f : 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) hidden[j][r] = fmaf(by_value, acc[r], fmaf(by_abs, fabsf(acc[r]), hidden[j][r]));
    });

    // 2. the w2 and offset blocks
    f32x4 dpre[MB];                            // adjoints of the hidden pre-activations, this lane's units
#pragma unroll
    for (int j = 0; j < MB; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) dpre[j][r] = 0.0f;
    lds_barrier();                             // every wave has finished with the block buffers
    stream.begin(a.frags + (size_t)(N + 1) * MB * Stream::kChunk, 2 * MB, buf);
    stream.template run<MB, 1>(st, bias_lds + (N + 1) * MB * 16, q_lds, N, [&](int, int j, int blk, const f32x4 &acc, float) {
        const int kind = blk / MB;             // 0: w2, 1: offset, beyond: padding of the last round of steps
        f32x4 first, second;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float pre = hidden[j][r], x = acc[r];
            const float hid = pre > 0.0f ? pre : expm1f(pre);
            const float d_pre = e * fabsf(x) * (pre > 0.0f ? 1.0f : expf(pre));
            const float d_gen2 = e * hid * (x > 0.0f ? 1.0f : x < 0.0f ? -1.0f : 0.0f);
            const float d_off = x > 0.0f ? e * gain[j][r] : 0.0f;
            first[r] = kind == 0 ? d_gen2 : d_off;
            second[r] = kind == 0 ? d_pre : e * fmaxf(x, 0.0f);
            dpre[j][r] = kind == 0 ? d_pre : dpre[j][r];
        }
        const uint32_t unit = 16 * j + 4 * q4, keep = kind < 2 ? drop : kDrop;
        store4(first, (kind == 0 ? (N + 1) * M : (N + 2) * M) + unit, keep);
        store4(second, (kind == 0 ? N * M : F) + unit, keep);
    });
    if (q4 == 0) {
        if constexpr (P == 1)
            __builtin_amdgcn_raw_buffer_store_b16(__builtin_bit_cast(uint16_t, (__bf16)e), dgen_buf, ((row_at + F + M) * 2u) | drop, 0, 0);
        else
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, e), dgen_buf, ((row_at + F + M) * 4u) | drop, 0, 0);
    }

    // 3. the agents' blocks again
    lds_barrier();
    stream.begin(a.frags, N * MB, buf);
    float share = 0.0f;                        // of dL/dq[n]: over this lane's units
    const uint32_t gq_row = (uint32_t)min(row[0], a.rows - 1) * (uint32_t)N;
    stream.template run<MB, 1>(st, bias_lds, q_lds, N, [&](int, int j, int blk, const f32x4 &acc, float qn) {
        f32x4 v;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const float x = acc[r];
            v[r] = dpre[j][r] * qn * (x > 0.0f ? 1.0f : x < 0.0f ? -1.0f : 0.0f);
            share = fmaf(dpre[j][r], fabsf(x), share);
        }
        const uint32_t keep = blk < N * MB ? drop : kDrop;
        store4(v, 16 * blk + 4 * q4, keep);
        if (j == MB - 1) {                     // the agent's last block: its row sum is complete
            float sum = share;
            sum += __shfl_xor(sum, 16);
            sum += __shfl_xor(sum, 32);
            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, sum), gq_buf,
                                                  ((gq_row + (uint32_t)(blk / MB)) * 4u) | (q4 == 0 ? keep : kDrop), 0, 0);
            share = 0.0f;
        }
    });
}

template <int MB, int P, int KS, int W>
hipError_t mixer_back_stream_launch(const MixerBackArgs &a, hipStream_t stream)
{
    const dim3 grid((unsigned)((a.rows + 16 * W - 1) / (16 * W))), block(64 * W);
    const size_t lds = BlockStream<P, KS, W>::kLdsBytes + sizeof(float) * ((size_t)a.F + (size_t)W * a.N * 16);
    hipError_t err = allow_large_lds<mixer_back_stream_kernel<MB, P, KS, W>>(kLdsLimit);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((mixer_back_stream_kernel<MB, P, KS, W>), grid, block, lds, stream, a);
    return hipGetLastError();
}

template <int P, int KS>
hipError_t mixer_back_stream_dispatch(int mb, const MixerBackArgs &a, hipStream_t stream)
{
    const bool big = mixer_big_shape_fits<P, KS>() && a.rows >= 8192;
    if constexpr (mixer_big_shape_fits<P, KS>()) {
        if (big) {
            switch (mb) {
            case 1: return mixer_back_stream_launch<1, P, KS, 8>(a, stream);
            case 2: return mixer_back_stream_launch<2, P, KS, 8>(a, stream);
            case 4: return mixer_back_stream_launch<4, P, KS, 8>(a, stream);
            default: return hipErrorInvalidValue;
            }
        }
    }
    switch (mb) {
    case 1: return mixer_back_stream_launch<1, P, KS, 4>(a, stream);
    case 2: return mixer_back_stream_launch<2, P, KS, 4>(a, stream);
    case 4: return mixer_back_stream_launch<4, P, KS, 4>(a, stream);
    default: return hipErrorInvalidValue;
    }
}

struct MixerGradPlan {
    int ldd, chunk;
    size_t off_dgen, off_partial, partial_bytes, bytes;
};

MixerGradPlan mixer_grad_plan(const marl_mixer_desc &d, int B, int T)
{
    MixerGradPlan p{};
    const long R = (long)B * T;
    const int F = (d.n_agents + 3) * d.embed;
    // whole 16-byte pieces, and eight columns from the last product's first one on (it takes the last embed + 1)
    p.ldd = F + (d.embed + 1 + 7) / 8 * 8;
    // few samples (B T, not B T N) and many products that run side by side: chunks of about 256 transitions
    const long chunks = std::max<long>(1, std::min<long>(256, R / 256));
    p.chunk = (int)(((R + chunks - 1) / chunks + 63) / 64 * 64);
    size_t off = 0;
    p.off_dgen = off;    off = (off + (size_t)R * p.ldd * 4 + 255) / 256 * 256;
    // room for sixteen of the largest partial results: the products run sixteen at a time
    p.partial_bytes = 16 * tn_partial_bytes(R, p.chunk, 384, 144);
    p.off_partial = off; off = (off + p.partial_bytes + 255) / 256 * 256;
    p.bytes = off;
    return p;
}

}  // namespace
}  // namespace marl

extern "C" {

int marl_mixer_grad_workspace_bytes(const marl_mixer *m, int32_t B, int32_t T, size_t *bytes)
{
    if (!m || !bytes) return MARL_ERR_NULL;
    const int F = (m->desc.n_agents + 3) * m->desc.embed;
    if (B < 1 || T < 1 || (int64_t)B * T * (F + m->desc.embed + 8) >= (int64_t)1 << 30) return MARL_ERR_BAD_DIM;
    *bytes = marl::mixer_grad_plan(m->desc, B, T).bytes;
    return MARL_OK;
}

int marl_mixer_grad(marl_mixer *m, int32_t B, int32_t T, const float *state, const float *q_taken,
                    const float *grad_q_total, void *workspace, size_t workspace_bytes, float *grad_q_taken,
                    float *grad_weights, void *hip_stream)
{
    if (!m) return MARL_ERR_NULL;
    size_t need = 0;
    const int rc = marl_mixer_grad_workspace_bytes(m, B, T, &need);
    if (rc != MARL_OK) return rc;
    if (!state || !q_taken || !grad_q_total || !workspace || !grad_q_taken || !grad_weights) return MARL_ERR_NULL;
    if (workspace_bytes < need) return MARL_ERR_BAD_DIM;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return MARL_ERR_BAD_ARG;
    marl::MixerDeviceGuard guard(m->desc.device);
    if (!guard.ok) return marl::report_device_error(hipErrorInvalidDevice, "hipSetDevice");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const marl::MixerGradPlan plan = marl::mixer_grad_plan(m->desc, B, T);
    const int N = m->desc.n_agents, M = m->desc.embed, S = m->desc.state_dim, F = (N + 3) * M;
    const long R = (long)B * T;
    char *dgen = static_cast<char *>(workspace) + plan.off_dgen;
    const bool dgen_bf16 = m->planes == 1;
    const size_t elem = dgen_bf16 ? 2 : 4;
    float *partial = reinterpret_cast<float *>(static_cast<char *>(workspace) + plan.off_partial);

    marl::MixerBackArgs a{};
    a.frags = m->frags; a.bias = m->bias; a.v2 = m->v2;
    a.N = N; a.M = M; a.S = S; a.ks = m->ks; a.rows = (int)R; a.T = T; a.F = F; a.ldd = plan.ldd;
    a.state = state; a.q = q_taken; a.e = grad_q_total; a.dgen = dgen; a.grad_q = grad_q_taken;
    hipError_t err = hipErrorInvalidValue;
    const int mb = M / 16;
#define MARL_MIXBACK_KS(PL)                                                                               \
    switch (m->ks) {                                                                                      \
    case 2: err = marl::mixer_back_stream_dispatch<PL, 2>(mb, a, stream); break;                          \
    case 4: err = marl::mixer_back_stream_dispatch<PL, 4>(mb, a, stream); break;                          \
    case 6: err = marl::mixer_back_stream_dispatch<PL, 6>(mb, a, stream); break;                          \
    case 8: err = marl::mixer_back_stream_dispatch<PL, 8>(mb, a, stream); break;                          \
    case 16: err = marl::mixer_back_stream_dispatch<PL, 16>(mb, a, stream); break;                        \
    default: break;                                                                                       \
    }
    if (m->planes == 2) {
        MARL_MIXBACK_KS(2);
    } else if (m->ks == 32) {
        err = marl::mixer_back_stream_dispatch<1, 32>(mb, a, stream);
    } else {
        MARL_MIXBACK_KS(1);
    }
#undef MARL_MIXBACK_KS
    if (err == hipSuccess) err = hipGetLastError();
    if (err != hipSuccess) return marl::report_device_error(err, "marl_mixer_grad launch");

    // parameter gradients: packed order Hw1 [N M, S], hb1, Hb1 [M, S], hbb1, Hw2 [M, S], hb2, V1 [M, S], c1, v2, c2
    float *gHw1 = grad_weights, *ghb1 = gHw1 + (size_t)N * M * S, *gHb1 = ghb1 + (size_t)N * M, *ghbb1 = gHb1 + (size_t)M * S;
    float *gHw2 = ghbb1 + M, *ghb2 = gHw2 + (size_t)M * S, *gV1 = ghb2 + M, *gc1 = gV1 + (size_t)M * S, *gv2 = gc1 + M;
    const marl::RowMap plain{dgen, 0, (int)R, plan.ldd, dgen_bf16 ? 1 : 0};
    const marl::RowMap states{state, (long)(T + 1) * S, T, S, 0};
    // one matrix: rows [r0, r0 + P) of it are adjoint columns [col0 + r0, ..); state columns in slices, the
    // column of ones (the bias) rides with the last slice
    std::vector<marl::TnProduct> products;
    auto matrix = [&](int col0, int rows_total, float *dst_w, float *dst_b) {
        const bool wide = rows_total > 128;
        const int p_step = wide ? 384 : 128, q_step = wide ? 128 : 320;
        for (int r0 = 0; r0 < rows_total; r0 += p_step)
            for (int k0 = 0; k0 < S; k0 += q_step) {
                const int P = std::min(p_step, rows_total - r0), Q = std::min(q_step, S - k0);
                const bool last = k0 + q_step >= S;
                marl::RowMap ar = plain, br = states;
                ar.base = dgen + (size_t)(col0 + r0) * elem;
                br.base = state + k0;
                products.push_back({ar, br, P, Q, last ? marl::kExtraOnes : marl::kExtraNone, last ? 1 : 0, 1, 0, S,
                                    dst_w + (size_t)r0 * S + k0, dst_b + r0});
            }
    };
    matrix(0, N * M, gHw1, ghb1);
    matrix(N * M, M, gHb1, ghbb1);
    matrix((N + 1) * M, M, gHw2, ghb2);
    matrix((N + 2) * M, M, gV1, gc1);
    {        // v2 and c2: the last M + 1 adjoint columns against the column of ones alone
        marl::RowMap ar = plain;
        ar.base = dgen + (size_t)F * elem;
        products.push_back({ar, states, M + 1, 0, marl::kExtraOnes, 1, 1, 0, 1, gv2, gv2});
    }
    err = marl::launch_tn_products(m->planes, products.data(), (int)products.size(), R, plan.chunk, partial, plan.partial_bytes, stream);
    if (err != hipSuccess) return marl::report_device_error(err, "marl_mixer_grad products");
    return MARL_OK;
}

namespace {
int mixer_update(marl_mixer *m, float *weights, const float *grad_weights, float lr, const marl::UpdateRule &rule, void *hip_stream)
{
    marl::MixerDeviceGuard guard(m->desc.device);
    if (!guard.ok) return marl::report_device_error(hipErrorInvalidDevice, "hipSetDevice");
    const size_t n_params = marl::mixer_params(&m->desc);
    const size_t N = m->desc.n_agents, M = m->desc.embed, S = m->desc.state_dim, F = (N + 3) * M;
    if (!m->repack_map) {
        size_t bytes = 0, frag_bytes = 0;
        {
            std::vector<float> zeros(n_params, 0.0f);
            char *host = marl::pack_mixer_image(m->desc, zeros.data(), &bytes, &frag_bytes);
            if (!host) return MARL_ERR_NOMEM;
            std::free(host);
        }
        std::vector<int32_t> map;
        const size_t frag_elems = frag_bytes / 2;
        const bool ok = marl::probe_fragment_map(n_params, frag_elems, [&](const float *w, uint16_t *out) {
            size_t b2, f2;
            char *host = marl::pack_mixer_image(m->desc, w, &b2, &f2);
            if (!host) return false;
            std::memcpy(out, host, frag_elems * 2);
            std::free(host);
            return true;
        }, &map);
        if (!ok) return MARL_ERR_NOMEM;
        // the tables are copies: hb1 | hbb1 | hb2 | c1, then v2, then c2 (packed order of the parameters:
        // Hw1, hb1, Hb1, hbb1, Hw2, hb2, V1, c1, v2, c2)
        const size_t o_hb1 = N * M * S, o_hbb1 = o_hb1 + N * M + M * S, o_hb2 = o_hbb1 + M + M * S, o_c1 = o_hb2 + M + M * S;
        const size_t o_v2 = o_c1 + M, o_c2 = o_v2 + M;
        for (size_t i = 0; i < N * M; ++i) map.push_back((int32_t)(o_hb1 + i));
        for (size_t i = 0; i < M; ++i) map.push_back((int32_t)(o_hbb1 + i));
        for (size_t i = 0; i < M; ++i) map.push_back((int32_t)(o_hb2 + i));
        for (size_t i = 0; i < M; ++i) map.push_back((int32_t)(o_c1 + i));
        for (size_t i = 0; i < M; ++i) map.push_back((int32_t)(o_v2 + i));
        map.push_back((int32_t)o_c2);
        int32_t *dev = nullptr;
        hipError_t err = hipMalloc(&dev, map.size() * sizeof(int32_t));
        if (err != hipSuccess) return err == hipErrorOutOfMemory ? MARL_ERR_NOMEM : marl::report_device_error(err, "hipMalloc");
        err = hipMemcpy(dev, map.data(), map.size() * sizeof(int32_t), hipMemcpyHostToDevice);
        if (err != hipSuccess) { (void)hipFree(dev); return marl::report_device_error(err, "hipMemcpy"); }
        m->repack_map = dev;
        m->frag_elems = frag_elems;
        m->table_entries = F + M + 1;
    }
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipError_t err = marl::launch_sgd_and_fragments(weights, grad_weights, lr, n_params, m->repack_map, m->frag_elems, m->image, stream, rule);
    if (err == hipSuccess)
        err = marl::launch_copy_refresh(weights, m->repack_map + m->frag_elems, m->table_entries, const_cast<float *>(m->bias), stream);
    if (err != hipSuccess) return marl::report_device_error(err, "mixer update launch");
    return MARL_OK;
}
bool finite_value(float v) { return v == v && v - v == 0.0f; }
}  // namespace

int marl_mixer_sgd_step(marl_mixer *m, float *weights, const float *grad_weights, float lr, void *hip_stream)
{
    if (!m || !weights || !grad_weights) return MARL_ERR_NULL;
    if (!finite_value(lr)) return MARL_ERR_BAD_ARG;
    return mixer_update(m, weights, grad_weights, lr, marl::UpdateRule(), hip_stream);
}

int marl_mixer_rmsprop_step(marl_mixer *m, float *weights, const float *grad_weights, float *sq_avg, float lr, float alpha,
                            float eps, void *hip_stream)
{
    if (!m || !weights || !grad_weights || !sq_avg) return MARL_ERR_NULL;
    if (!finite_value(lr) || !(alpha >= 0.0f && alpha <= 1.0f) || !(eps > 0.0f) || !finite_value(eps)) return MARL_ERR_BAD_ARG;
    marl::UpdateRule rule;
    rule.sq_avg = sq_avg; rule.alpha = alpha; rule.eps = eps;
    return mixer_update(m, weights, grad_weights, lr, rule, hip_stream);
}

}  // extern "C"
