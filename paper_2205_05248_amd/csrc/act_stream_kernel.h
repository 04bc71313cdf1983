// Streaming decision-step kernel for gfx950 on items of 16 (env, agent) rows.
//
// The decision step reads every input once and reuses nothing, so it is bound by memory traffic
// and its whole job is to keep enough of it in flight.  This kernel is built around that:
//
//   * One workgroup per compute unit (two for hidden 64), one wavefront per block of 16 hidden
//     units.  Every wave holds its block's rows of W1, W_ih and W_hh in registers for the whole
//     launch (fc2 sits in LDS), so that a matrix product never reads a weight from LDS; every wave
//     does the same work in every step, which keeps the four SIMDs evenly loaded.
//   * Inputs travel global memory -> LDS directly (buffer loads with the LDS modifier): they cost
//     no registers while in flight, all waves issue them, and a ring of three raw items per
//     stream keeps two items (about 56 KB per compute unit for the largest workload) on their way
//     while a third is being consumed.  Buffer descriptors bound every array: rows past the
//     end read zeros and their stores are dropped by the hardware, so there is no tail code.
//   * Items are dealt round-robin over the workgroups (item k of workgroup g is g + k G): at
//     any moment the chip reads one contiguous front of memory instead of G distant streams.
//   * The item's work is pipelined over the steps, one LDS-only barrier per step.  In step s
//         issue    observations, availability, step counters of item s + 4; incoming state of item s + 2
//         convert  item s + 2: fp32 observations -> bf16 operand fragments (+ the agent id columns),
//                  availability bytes -> a bit mask per row
//         fc1      item s + 1: x = ReLU(W1 [o, id] + b1)              (this wave's 16 units)
//         GRU      item s: both products, gates, h' -> global memory and LDS (this wave's 16 units)
//         fc2      item s - 1: Q block, store, masked argmax          (waves 0 .. ceil(A/16) - 1)
//         choose   item s - 3: greedy or explored action, store       (last wave)
//     and every fourth step one wave makes the epsilon-greedy draws for four items (64 rows) at once.
//
// A wait for the loads counts vector-memory instructions (s_waitcnt vmcnt), so every wave issues
// exactly the same number of them in every step, unconditionally: what does not apply goes out
// with an offset beyond its descriptor.  No load inside the loop has a register as destination.
#pragma once
#include <hip/hip_runtime.h>

#include <atomic>
#include <type_traits>

#include "fused16.h"

namespace marl {

namespace {

typedef __attribute__((address_space(3))) char lds_char;

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr uint32_t kDropOffset = 0xFFFFFFF0u;       // beyond any descriptor: loads give zero, stores vanish
// The same for a lane that never takes part, as a term of a sum: every array is below 2^30 bytes, so adding any
// real offset to it stays beyond the descriptor without wrapping round.  No comparison, no mask kept in registers.
constexpr uint32_t kDeadLane = 0x80000000u;
constexpr int kNonTemporal = 2;                     // cache policy of the streamed loads and stores

template <int H, int P> struct Stream16 {
    static constexpr int NW = H / 16;               // waves = blocks of 16 hidden units
    static constexpr int KS = H / 32;               // k-steps over the hidden layer
    static constexpr int KM = 48 / (4 * P);         // first-layer k-steps whose fragments fit 48 registers
    static constexpr int kFrag = P * 1024;
};

// Byte offsets of the LDS buffers.  Everything whose size does not depend on the observation width
// comes first, at compile-time offsets (an LDS access then needs no address arithmetic beyond its
// lane's own constant); the ring of raw observations is last.
template <int H, int P> struct StreamLds {
    static constexpr int KS = H / 32, KM = Stream16<H, P>::KM, kFrag = Stream16<H, P>::kFrag;
    static constexpr int obs_frags = 0;                                 // [2][KM][P][1024], k-steps past the first layer's width zero
    static constexpr int x_frags = obs_frags + 2 * KM * kFrag;          // [2][KS][P][1024]
    static constexpr int hp_frags = x_frags + 2 * KS * kFrag;           // [2][KS][P][1024]
    static constexpr int w2 = hp_frags + 2 * KS * kFrag;                // [4][KS][P][1024]
    static constexpr int bias = w2 + 4 * KS * kFrag;                    // [5][H] floats: b1, b_ir + b_hr, b_iz + b_hz, b_in, b_hn; then b2 [64]
    static constexpr int bits = bias + (5 * H + 64) * 4;                // [8][16] u64: a row's available actions
    static constexpr int flags = bits + 8 * 16 * 8;                     // [8][64] u32: reset flag of the row's environment
    static constexpr int stept = flags + 8 * 256;                       // [8][64] i32
    static constexpr int rng = stept + 8 * 256;                         // [2][64] {explore, pick bits}
    static constexpr int cand = rng + 2 * 64 * 8;                       // [4][4][16] {best q, best index}
    static constexpr int dump = cand + 4 * 4 * 16 * 8;                  // [1024] target of loads that do not apply
    // the raw state: KiB chunks (what one load instruction brings) kHChunk apart, so that the rows of different chunks
    // start in different banks (rows are 4 H bytes: a whole number of times round the banks)
    static constexpr int kHChunk = 1024 + 32, kHSlot = (64 * H / 1024) * kHChunk;
    static constexpr int raw_h = dump + 1024;                           // [3][kHSlot]
    static constexpr int raw_avail = raw_h + 3 * kHSlot;                // [3][1024]
    static constexpr int raw_obs = raw_avail + 3 * 1024;                // [3][obs_slot]
    static_assert(bits % 16 == 0 && raw_h % 16 == 0, "alignment of the 64-bit tables and of the load targets");
    __host__ __device__ static constexpr int obs_slot(int D) { return (64 * D + 1023) / 1024 * 1024; }    // one raw item, whole KiB
    __host__ __device__ static constexpr int total(int D) { return raw_obs + 3 * obs_slot(D); }
};

constexpr int vmcnt_imm(int n) { return (n & 15) | (7 << 4) | (15 << 8) | ((n >> 4) << 14); }

// The step's barrier: this wave's LDS writes are done, then wait for the workgroup.  It must not be
// the fenced barrier the other kernels use: a fence on LDS also waits for every load that is on its
// way into LDS, which is exactly what has to stay in flight across steps.
__device__ __forceinline__ void step_barrier()
{
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

}  // namespace

struct ActStreamArgs {
    NetFrags net;
    int rows;                   // E * N
    int n_items;                // ceil(rows / 16)
    int E;
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

// Eight consecutive floats from a 4-byte aligned LDS address.  Written out as instructions: the compiler would pair
// such reads up, and it makes a paired read of memory that loads are on their way into wait for every one of them.
__device__ __forceinline__ void lds_read8(uint32_t addr, float (&v)[8])
{
    asm volatile("ds_read_b32 %0, %8\n\tds_read_b32 %1, %8 offset:4\n\tds_read_b32 %2, %8 offset:8\n\tds_read_b32 %3, %8 offset:12\n\t"
                 "ds_read_b32 %4, %8 offset:16\n\tds_read_b32 %5, %8 offset:20\n\tds_read_b32 %6, %8 offset:24\n\tds_read_b32 %7, %8 offset:28\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&v"(v[0]), "=&v"(v[1]), "=&v"(v[2]), "=&v"(v[3]), "=&v"(v[4]), "=&v"(v[5]), "=&v"(v[6]), "=&v"(v[7])
                 : "v"(addr)
                 : "memory");
}

// A copy of a per-lane value that the compiler cannot trace back to its source.  What is derived from the copy
// inside a block that only one wave runs is computed there, when that wave gets there, instead of being kept in
// registers of every wave for the whole launch.
__device__ __forceinline__ int opaque(int v)
{
    asm volatile("" : "+v"(v));
    return v;
}

// OPS: observation loads per wave and item (ceil(KiB of an item's observations / waves)); QV: n_actions is a multiple of four
// (a lane's four Q values go out as one 16-byte store).
template <int H, int P, int OPS, bool QV>
__global__ __launch_bounds__(64 * (H / 16), 2) void act_stream_kernel(const ActStreamArgs args)
{
    using Sh = Stream16<H, P>;
    using L = StreamLds<H, P>;
    constexpr int NW = Sh::NW, KS = Sh::KS, KM = Sh::KM, GR = KM / 3, kFrag = Sh::kFrag;
    constexpr int CJ = (KM + NW - 1) / NW;                     // first-layer k-steps a wave converts per item, at most
    constexpr int kBitsWave = NW - 2, kDrawWave = NW - 3, kChooseWave = NW - 1;
    constexpr int kQWave0 = NW == 8 ? 3 : 0;                  // action block ab is wave kQWave0 + ab's (the first waves convert two k-steps)
    extern __shared__ __attribute__((aligned(16))) char lds[];
    const NetFrags &net = args.net;
    const int N = net.N, D = net.D, A = net.A;
    const int ks1 = (D + N + 31) / 32;              // first-layer k-steps, agent id columns included
    const int AB = (A + 15) / 16;
    const int obs_slot = L::obs_slot(D);
    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int rows = args.rows;
    const int count = (args.n_items - (int)blockIdx.x + (int)gridDim.x - 1) / (int)gridDim.x;       // items of this workgroup, >= 1
    const uint32_t stride16 = gridDim.x * 16u;                  // rows from one item of this workgroup to its next
    // row / N by a multiplication (rows < 2^22, N <= 64: exact); N = 1 has no 32-bit multiplier
    const uint32_t n_magic = N > 1 ? (uint32_t)(0x100000000ull / (uint32_t)N) + 1u : 0u;
    auto env_of = [&](uint32_t row) { return N > 1 ? __umulhi(row, n_magic) : row; };

    // ---- descriptors (sizes in bytes; the host has checked that every one is below 2^30)
    const __amdgpu_buffer_rsrc_t r_obs = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(args.obs), 0, rows * D * 4, kRawBuffer);
    const __amdgpu_buffer_rsrc_t r_h = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(args.h_in), 0, rows * H * 4, kRawBuffer);
    // the third load of a step: wave 0 availability (read four bytes at a time: the last word may reach up to
    // three bytes past the array), wave 1 step counters, wave 2 reset flags, the others nothing
    const __amdgpu_buffer_rsrc_t r_misc =
        w == 0   ? __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(args.avail), 0, (rows * A + 3) & ~3, kRawBuffer)
        : w == 1 ? __builtin_amdgcn_make_buffer_rsrc(const_cast<int32_t *>(args.step_t), 0, args.E * 4, kRawBuffer)
                 : __builtin_amdgcn_make_buffer_rsrc(const_cast<uint8_t *>(args.reset), 0, w == 2 && args.reset ? args.E : 0, kRawBuffer);
    const __amdgpu_buffer_rsrc_t r_ho = __builtin_amdgcn_make_buffer_rsrc(args.h_out, 0, rows * H * 4, kRawBuffer);
    const __amdgpu_buffer_rsrc_t r_q = __builtin_amdgcn_make_buffer_rsrc(args.q_out, 0, args.q_out ? rows * A * 4 : 0, kRawBuffer);
    const __amdgpu_buffer_rsrc_t r_ac = __builtin_amdgcn_make_buffer_rsrc(args.action, 0, rows * 4, kRawBuffer);

    const int n_chunks = (64 * D + 1023) / 1024;            // KiB of one item's observations: (OPS - 1) NW < n_chunks <= OPS NW
    constexpr int kOpsPerStep = OPS + 2 + 1 + (QV ? 1 : 4) + 1;     // vector-memory instructions of a wave in one step

    // ---- per-lane addresses that never change (LDS byte addresses; global byte offsets within an item).  Buffers sit
    // at compile-time offsets, so most accesses are one of these plus an immediate.
    const uint32_t lane16 = lane * 16;
    const uint32_t v_avail = lane < A ? lane16 : kDeadLane;                    // an item's availability: 16 A bytes
    const uint32_t a_bias = L::bias + (16 * w + 4 * q4) * 4;
    const uint32_t pub = (w / 2) * kFrag + lane16 + (w & 1) * 8;               // this wave's half of k-step w / 2
    const uint32_t a_hraw = L::raw_h + (c / (256 / H)) * L::kHChunk + (c % (256 / H)) * 4 * H + 16 * q4;
    const uint32_t a_hflag = L::flags + (w * (256 / H) + lane * 4 / H) * 4;    // the row whose state this lane loads
    const uint32_t g_hout = (c * H + 16 * w + 4 * q4) * 4;
    const uint32_t a_cr = L::raw_obs + c * 4 * D + (32 * w + 8 * q4) * 4;      // k-step w of the raw observations; k-step w + NW j: + 128 NW j
    const uint32_t a_cw = L::obs_frags + w * kFrag + lane16;                   // its fragment; + NW j kFrag

    // ---- loads of step s: observations, availability, step counters, reset flags of item s + 4; state of item s + 2.
    // A row whose environment starts an episode gets no load of its state: zeros land in LDS instead.
    // row_s = first row of item s; slot_*: ring positions of items s + 4 and s + 2.
    auto issue = [&](auto guard, int s, uint32_t row_s, int slot_o, int slot_h) {
        constexpr bool GUARD = decltype(guard)::value;       // item s + 2 may not exist (a step before the first item)
        const int ko = s + 4, kh = s + 2;
        const uint32_t row_o = row_s + 4 * stride16, row_h = row_s + 2 * stride16;
        uint32_t flag = 0;
        if (!GUARD || kh >= 0) flag = *reinterpret_cast<const uint32_t *>(lds + a_hflag + (kh & 7) * 256);
        const uint32_t base_o = row_o * (uint32_t)(4 * D);
        const int target = L::raw_obs + slot_o * obs_slot;
        // the observation loads, straight-line: chunks w, w + NW, ...; only the last can lie past the item, for some waves
#pragma unroll
        for (int j = 0; j < OPS; ++j) {
            const int chunk = w + NW * j;
            const bool live = j + 1 < OPS || chunk < n_chunks;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r_obs, (lds_char *)(lds + (live ? target + chunk * 1024 : L::dump)), 16,
                                                     base_o + chunk * 1024 + (live ? lane16 : kDeadLane), 0, 0, kNonTemporal);
        }
        if (w == 0) {
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r_misc, (lds_char *)(lds + (L::raw_avail + slot_o * 1024)), 16,
                                                     row_o * (uint32_t)A + v_avail, 0, 0, kNonTemporal);
        } else if (w <= 2) {     // the environment's step counter (wave 1) or reset flag (wave 2), one lane per row
            // a row past the end belongs to an environment past the last: its load finds nothing by itself
            const int l = opaque(lane);
            const uint32_t e = env_of(row_o + (l & 15));
            const uint32_t dead = l < 16 ? 0u : kDeadLane;
            if (w == 1) __builtin_amdgcn_raw_ptr_buffer_load_lds(r_misc, (lds_char *)(lds + (L::stept + (ko & 7) * 256)), 4, e * 4u + dead, 0, 0, 0);
            else __builtin_amdgcn_raw_ptr_buffer_load_lds(r_misc, (lds_char *)(lds + (L::flags + (ko & 7) * 256)), 1, e + dead, 0, 0, 0);
        } else {                 // the descriptor is empty
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r_misc, (lds_char *)(lds + L::dump), 1, kDropOffset, 0, 0, 0);
        }
        __builtin_amdgcn_raw_ptr_buffer_load_lds(r_h, (lds_char *)(lds + (L::raw_h + slot_h * L::kHSlot + w * L::kHChunk)), 16,
                                                 (!GUARD || kh >= 0) && (flag & 0xFFu) == 0 ? row_h * (uint32_t)(4 * H) + w * 1024 + lane16 : kDropOffset, 0, 0,
                                                 kNonTemporal);
    };

    // ---- resident weights of this wave's block of hidden units; k-steps past the first layer's width are zero
    WFrag<P> w1[KM], wih[3][KS], whh[3][KS];
#pragma unroll
    for (int ks = 0; ks < KM; ++ks) {
        w1[ks] = load_wfrag<P>(net.w1x_16 + ((size_t)(w * ks1 + min(ks, ks1 - 1)) * P) * 64 + lane);
        if (ks >= ks1) {
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                w1[ks].hi[i] = (__bf16)0.0f;
                if constexpr (P == 2) w1[ks].lo[i] = (__bf16)0.0f;
            }
        }
    }
#pragma unroll
    for (int gate = 0; gate < 3; ++gate)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            wih[gate][ks] = load_wfrag<P>(net.wih_16 + ((size_t)((gate * NW + w) * KS + ks) * P) * 64 + lane);
            whh[gate][ks] = load_wfrag<P>(net.whh_16 + ((size_t)((gate * NW + w) * KS + ks) * P) * 64 + lane);
        }
    // biases -> LDS: [b1, b_ir + b_hr, b_iz + b_hz, b_in, b_hn][H], then b2 [64]; the observation fragments' k-steps past
    // the first layer's width and the reset flags of items before the first are zero
    {
        float *bt = reinterpret_cast<float *>(lds + L::bias);
        const float *src[5] = {net.b1_plain, net.bias_r, net.bias_z, net.bias_in, net.bias_hn};
        for (int i = threadIdx.x; i < 5 * H; i += 64 * NW) bt[i] = src[i / H][i % H];
        for (int i = threadIdx.x; i < 64; i += 64 * NW) bt[5 * H + i] = i < 16 * AB ? net.b2[i] : 0.0f;
        uint32_t *of = reinterpret_cast<uint32_t *>(lds + L::obs_frags);
        for (int i = threadIdx.x; i < 2 * KM * kFrag / 4; i += 64 * NW) of[i] = 0u;
        uint32_t *fl = reinterpret_cast<uint32_t *>(lds + L::flags);
        for (int i = threadIdx.x; i < 8 * 64; i += 64 * NW) fl[i] = 0u;
    }
    // fc2 fragments -> LDS
    {
        const __amdgpu_buffer_rsrc_t r_w2 = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16x8 *>(net.w2_16), 0, AB * KS * P * 1024, kRawBuffer);
        for (int i = w; i < AB * KS * P; i += NW)
            __builtin_amdgcn_raw_ptr_buffer_load_lds(r_w2, (lds_char *)(lds + (L::w2 + i * 1024)), 16, i * 1024 + lane16, 0, 0, 0);
    }
    step_barrier();                              // the flags are cleared before the first loads land in them
    uint32_t row_s = ((uint32_t)blockIdx.x - 4u * gridDim.x) * 16u;       // first row of "item -4" (wraps; only sums with 4 stride16 are used)
    issue(std::true_type{}, -4, row_s, 0, 1);
    row_s += stride16;
    issue(std::true_type{}, -3, row_s, 1, 2);
    row_s += stride16;
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));
    step_barrier();

    auto lds_frag = [&](uint32_t addr) {         // one k-step's operand at a byte address (planes 1 KiB apart)
        Frag<P> fr;
        fr.hi = *reinterpret_cast<const bf16x8 *>(lds + addr);
        if constexpr (P == 2) fr.lo = *reinterpret_cast<const bf16x8 *>(lds + addr + 1024);
        return fr;
    };
    // this wave's units as its half of the next operand's k-step w / 2
    auto publish = [&](uint32_t addr, const f32x4 &v) {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        bf16x4 hi, lo;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            hi[r] = (__bf16)v[r];
            if constexpr (P == 2) lo[r] = (__bf16)(v[r] - (float)hi[r]);
        }
        *reinterpret_cast<bf16x4 *>(lds + addr) = hi;
        if constexpr (P == 2) *reinterpret_cast<bf16x4 *>(lds + addr + 1024) = lo;
    };
    auto pair_of = [](uint32_t lo, uint32_t hi) { return ((uint64_t)hi << 32) | lo; };

    // ring positions (0, 1, 2) of the items s + 4, s + 2 (= s + 5), s (= s + 3) of the step
    int ring_a = 2, ring_b = 0, ring_c = 1;      // s = -2: (s + 4) % 3, (s + 5) % 3, (s + 3) % 3

    // GUARD: a step near either end of the run, where some of the items s + 4 .. s - 3 do not exist
    auto step = [&](auto parity, auto guard, int s) {
        constexpr int PS = decltype(parity)::value;          // s & 1; items s + 2 and s share it, s + 1 and s - 1 have the other
        constexpr bool GUARD = decltype(guard)::value;
        issue(guard, s, row_s, ring_a, ring_b);
        // ------------------------------------------------------------ convert: item s + 2
        if (!GUARD || s + 2 < count) {
            const int k = s + 2;
            if (w == kBitsWave) {       // availability bytes of the row -> bit a = action a usable
                const int l = opaque(lane), lq = l >> 4, lc = l & 15;
                // the sixteen bytes from action 16 q on; what lies past the row's A bytes is masked afterwards
                const uint32_t at = L::raw_avail + ring_b * 1024 + lc * A + 16 * lq;
                uint32_t m = 0;
                if constexpr (QV) {
                    uint32_t word[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) word[i] = *reinterpret_cast<const uint32_t *>(lds + at + 4 * i);
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        // bit 7 of every non-zero byte, then the four of them moved to bits 0 .. 3
                        uint32_t t = (((word[i] & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | word[i]) & 0x80808080u;
                        t >>= 7;
                        t |= t >> 7;
                        t |= t >> 14;
                        m |= (t & 0xFu) << (4 * i);
                    }
                } else {
                    uint32_t byte[16];
#pragma unroll
                    for (int i = 0; i < 16; ++i) byte[i] = *reinterpret_cast<const uint8_t *>(lds + at + i);
#pragma unroll
                    for (int i = 0; i < 16; ++i) m |= byte[i] ? (1u << i) : 0u;
                }
                const int left = A - 16 * lq;                                      // actions from 16 q on
                m &= left >= 16 ? 0xFFFFu : left > 0 ? (1u << left) - 1u : 0u;
                const uint64_t part = (uint64_t)m << (16 * lq);
                const uint64_t all = ((uint64_t)or_quarters((uint32_t)(part >> 32)) << 32) | or_quarters((uint32_t)part);
                if (lq == 0) *reinterpret_cast<uint64_t *>(lds + L::bits + ((k & 7) * 16 + lc) * 8) = all;
            }
            const uint32_t slot = ring_b * obs_slot;
#pragma unroll
            for (int j = 0; j < CJ; ++j) {
                const int ks = w + NW * j;
                if (ks >= ks1) continue;
                float v[8];
                if ((D & 3) == 0) {                                   // rows are 16-byte aligned
                    const f32x4 *at = static_cast<const f32x4 *>(__builtin_assume_aligned(lds + a_cr + 128 * NW * j + slot, 16));
                    const f32x4 a = at[0], b = at[1];
#pragma unroll
                    for (int i = 0; i < 4; ++i) { v[i] = a[i]; v[4 + i] = b[i]; }
                } else {
                    lds_read8(a_cr + 128 * NW * j + slot, v);
                }
                Frag<P> fr = to_frag<P>(v);
                if (32 * ks + 32 > D) {
                    // positions from D on hold the one-hot agent id: whatever was read there is cleared (bit-wise, on the
                    // packed pairs) and the one at position D + n set
                    const int l = opaque(lane), lq = l >> 4, lc = l & 15;
                    const uint32_t row = row_s + 2 * stride16 + lc;
                    const int n = (int)(row - env_of(row) * (uint32_t)N);
                    const int past = D - (32 * ks + 8 * lq);       // how many of this lane's eight elements are observations
                    const int at = n + past;                        // where the one goes, if within 0 .. 7 and not before `past`
                    const uint32_t one = (at >= 0 && at >= past && at < 8) ? (0x3F80u << (16 * (at & 1))) : 0u;
                    u32x4_t hi = __builtin_bit_cast(u32x4_t, fr.hi);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const uint32_t keep = past >= 2 * r + 2 ? 0xFFFFFFFFu : past == 2 * r + 1 ? 0x0000FFFFu : 0u;
                        hi[r] = (hi[r] & keep) | ((at >> 1) == r ? one : 0u);
                        if constexpr (P == 2) {
                            u32x4_t lo = __builtin_bit_cast(u32x4_t, fr.lo);
                            lo[r] &= keep;
                            fr.lo = __builtin_bit_cast(bf16x8, lo);
                        }
                    }
                    fr.hi = __builtin_bit_cast(bf16x8, hi);
                }
                *reinterpret_cast<bf16x8 *>(lds + a_cw + (NW * j + PS * KM) * kFrag) = fr.hi;
                if constexpr (P == 2) *reinterpret_cast<bf16x8 *>(lds + a_cw + (NW * j + PS * KM) * kFrag + 1024) = fr.lo;
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // ------------------------------------------------------------ fc1: item s + 1
        if (!GUARD || (s + 1 >= 0 && s + 1 < count)) {
            constexpr int PB = (1 - PS) * KM * kFrag;
            // three groups of fragments, the reads of a group two groups ahead of its products
            Frag<P> ga[GR], gb[GR];
            f32x4 acc = *reinterpret_cast<const f32x4 *>(lds + a_bias);
#pragma unroll
            for (int i = 0; i < GR; ++i) ga[i] = lds_frag(L::obs_frags + lane16 + PB + i * kFrag);
#pragma unroll
            for (int i = 0; i < GR; ++i) gb[i] = lds_frag(L::obs_frags + lane16 + PB + (GR + i) * kFrag);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < GR; ++i) mma16<P>(acc, w1[i], ga[i]);
#pragma unroll
            for (int i = 0; i < GR; ++i) ga[i] = lds_frag(L::obs_frags + lane16 + PB + (2 * GR + i) * kFrag);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < GR; ++i) mma16<P>(acc, w1[GR + i], gb[i]);
#pragma unroll
            for (int i = 0; i < GR; ++i) mma16<P>(acc, w1[2 * GR + i], ga[i]);
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[r] = fmaxf(acc[r], 0.0f);
            publish(L::x_frags + pub + (1 - PS) * KS * kFrag, acc);
        }
        __builtin_amdgcn_sched_barrier(0);
        // ------------------------------------------------------------ GRU: item s
        f32x4 hv = {0.0f, 0.0f, 0.0f, 0.0f};
        uint32_t h_off = kDropOffset;
        if (!GUARD || (s >= 0 && s < count)) {
            const uint32_t hr = a_hraw + ring_c * L::kHSlot;
            // LDS reads run two k-steps ahead of the products that use them
            f32x4 ha[2], hb4[2];
            Frag<P> x[2];
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                // the operand's k order: features 32 ks + 4 q + 0..3, then 32 ks + 16 + 4 q + 0..3
                ha[ks] = *reinterpret_cast<const f32x4 *>(lds + hr + 128 * ks);
                hb4[ks] = *reinterpret_cast<const f32x4 *>(lds + hr + 128 * ks + 64);
                x[ks] = lds_frag(L::x_frags + lane16 + (PS * KS + ks) * kFrag);
            }
            f32x4 acc_r = *reinterpret_cast<const f32x4 *>(lds + a_bias + 4 * H), acc_z = *reinterpret_cast<const f32x4 *>(lds + a_bias + 8 * H);
            f32x4 acc_in = *reinterpret_cast<const f32x4 *>(lds + a_bias + 12 * H), acc_hn = *reinterpret_cast<const f32x4 *>(lds + a_bias + 16 * H);
            hv = *reinterpret_cast<const f32x4 *>(lds + hr + 64 * w);          // this wave's own units of the old state
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const float v[8] = {ha[ks & 1][0], ha[ks & 1][1], ha[ks & 1][2], ha[ks & 1][3],
                                    hb4[ks & 1][0], hb4[ks & 1][1], hb4[ks & 1][2], hb4[ks & 1][3]};
                const Frag<P> hb = to_frag<P>(v);
                const Frag<P> xk = x[ks & 1];
                if (ks + 2 < KS) {
                    ha[ks & 1] = *reinterpret_cast<const f32x4 *>(lds + hr + 128 * (ks + 2));
                    hb4[ks & 1] = *reinterpret_cast<const f32x4 *>(lds + hr + 128 * (ks + 2) + 64);
                    x[ks & 1] = lds_frag(L::x_frags + lane16 + (PS * KS + ks + 2) * kFrag);
                }
                mma16<P>(acc_r, wih[0][ks], xk);
                mma16<P>(acc_z, wih[1][ks], xk);
                mma16<P>(acc_in, wih[2][ks], xk);
                mma16<P>(acc_r, whh[0][ks], hb);
                mma16<P>(acc_z, whh[1][ks], hb);
                mma16<P>(acc_hn, whh[2][ks], hb);
                __builtin_amdgcn_sched_barrier(0);
            }
            hv = gru_blend4(acc_r, acc_z, acc_in, acc_hn, hv);
            h_off = row_s * (uint32_t)(4 * H) + g_hout;
            publish(L::hp_frags + pub + PS * KS * kFrag, hv);
        }
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, hv), r_ho, h_off, 0, kNonTemporal);
        __builtin_amdgcn_sched_barrier(0);
        // ------------------------------------------------------------ fc2: item s - 1, one action block per wave
        f32x4 qv = {0.0f, 0.0f, 0.0f, 0.0f};
        uint32_t q_off = kDropOffset;
        if ((!GUARD || (s - 1 >= 0 && s - 1 < count)) && w >= kQWave0 && w < kQWave0 + AB) {
            const int ab = w - kQWave0;
            const int k = s - 1;
            const int l = opaque(lane), lq = l >> 4, lc = l & 15;
            const uint32_t at = l * 16;
            Frag<P> hb[KS];
            WFrag<P> wf[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                hb[ks] = lds_frag(L::hp_frags + at + ((1 - PS) * KS + ks) * kFrag);
                const Frag<P> t = lds_frag(L::w2 + ab * KS * kFrag + at + ks * kFrag);
                wf[ks].hi = t.hi;
                if constexpr (P == 2) wf[ks].lo = t.lo;
            }
            const int a0 = 16 * ab + 4 * lq;
            qv = *reinterpret_cast<const f32x4 *>(lds + L::bias + 20 * H + a0 * 4);
            const uint64_t bits = *reinterpret_cast<const uint64_t *>(lds + L::bits + ((k & 7) * 16 + lc) * 8);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) mma16<P>(qv, wf[ks], hb[ks]);
            q_off = ((row_s - stride16 + lc) * (uint32_t)A + a0) * 4u + (a0 < A ? 0u : kDeadLane);
            const uint32_t slots = (uint32_t)(bits >> a0) & 0xFu;
            float best_q = 0.0f;
            int best = -1;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const bool ok = (slots >> r) & 1u;
                if (ok && (best < 0 || qv[r] > best_q)) { best_q = qv[r]; best = a0 + r; }
            }
            auto better = [](float qa, int ia, float qb, int ib, float &q_out, int &i_out) {      // ties: the lower index
                const bool take_b = ib >= 0 && (ia < 0 || qb > qa || (qb == qa && ib < ia));
                q_out = take_b ? qb : qa;
                i_out = take_b ? ib : ia;
            };
            LanePair pq = halves16(__float_as_uint(best_q)), pi = halves16((uint32_t)best);
            better(__uint_as_float(pq.lower), (int)pi.lower, __uint_as_float(pq.upper), (int)pi.upper, best_q, best);
            pq = halves32(__float_as_uint(best_q));
            pi = halves32((uint32_t)best);
            better(__uint_as_float(pq.lower), (int)pi.lower, __uint_as_float(pq.upper), (int)pi.upper, best_q, best);
            if (lq == 0) *reinterpret_cast<uint64_t *>(lds + L::cand + (((k & 3) * 4 + ab) * 16 + lc) * 8) = pair_of(__float_as_uint(best_q), (uint32_t)best);
        }
        if constexpr (QV) {
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, qv), r_q, q_off, 0, kNonTemporal);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(qv[r]), r_q,
                                                      q_off != kDropOffset && 16 * (w - kQWave0) + 4 * q4 + r < A ? q_off + 4 * r : kDropOffset, 0, kNonTemporal);
        }
        __builtin_amdgcn_sched_barrier(0);
        // ------------------------------------------------------------ draws for items s - 2 .. s + 1, every fourth step
        if (((s - 2) & 3) == 0 && w == kDrawWave) {
            const int l = opaque(lane), lq = l >> 4, lc = l & 15;
            const int k = s - 2 + lq;
            const uint32_t row = row_s + (uint32_t)(lq - 2) * stride16 + lc;
            const int32_t t = *reinterpret_cast<const int32_t *>(lds + L::stept + (k & 7) * 256 + lc * 4);
            const uint32_t e = env_of(row);
            const ExploreDraw d = explore_draw(args.seed, e, row - e * (uint32_t)N, (uint32_t)t);
            *reinterpret_cast<uint64_t *>(lds + L::rng + ((((s - 2) >> 2) & 1) * 64 + l) * 8) = pair_of(d.u < args.epsilon ? 1u : 0u, d.pick_bits);
        }
        // ------------------------------------------------------------ choose: item s - 3
        int pick = 0;
        uint32_t a_off = kDropOffset;
        if ((!GUARD || (s - 3 >= 0 && s - 3 < count)) && w == kChooseWave) {
            const int k = s - 3;
            const int l = opaque(lane), lq = l >> 4, lc = l & 15;
            const uint64_t bits = *reinterpret_cast<const uint64_t *>(lds + L::bits + ((k & 7) * 16 + lc) * 8);
            const uint64_t draw = *reinterpret_cast<const uint64_t *>(lds + L::rng + (((k >> 2) & 1) * 64 + (k & 3) * 16 + lc) * 8);
            uint64_t cd[4];
#pragma unroll
            for (int ab = 0; ab < 4; ++ab) cd[ab] = *reinterpret_cast<const uint64_t *>(lds + L::cand + (((k & 3) * 4 + ab) * 16 + lc) * 8);
            float best_q = 0.0f;
            int best = -1;
#pragma unroll
            for (int ab = 0; ab < 4; ++ab) {     // blocks come in index order: a later one must be strictly better
                const float cq = __uint_as_float((uint32_t)cd[ab]);
                const int ci = (int)(uint32_t)(cd[ab] >> 32);
                if (ab < AB && ci >= 0 && (best < 0 || cq > best_q)) { best_q = cq; best = ci; }
            }
            pick = max(best, 0);
            if ((uint32_t)draw) {
                const uint32_t n_avail = (uint32_t)__popcll(bits);
                const uint32_t j = (uint32_t)(((uint64_t)(uint32_t)(draw >> 32) * (uint64_t)n_avail) >> 32);
                pick = n_avail ? nth_set_bit(bits, j) : 0;
            }
            a_off = (row_s - 3 * stride16 + lc) * 4u + (lq == 0 ? 0u : kDeadLane);
        }
        __builtin_amdgcn_raw_buffer_store_b32((uint32_t)pick, r_ac, a_off, 0, kNonTemporal);
        // everything issued before this step's instructions has landed once at most one step's worth is outstanding
        __builtin_amdgcn_s_waitcnt(vmcnt_imm(kOpsPerStep));
        step_barrier();
        const int t = ring_a;
        ring_a = ring_b; ring_b = ring_c; ring_c = t;
        row_s += stride16;
    };
    // steps -2 .. 2 (items before the first missing), 3 .. count - 3 (every item of the step exists), count - 2 .. count + 2
    using Even = std::integral_constant<int, 0>;
    using Odd = std::integral_constant<int, 1>;
    int s = -2;
    for (; s < 3 && s <= count + 2; ++s) {
        if (s & 1) step(Odd{}, std::true_type{}, s);
        else step(Even{}, std::true_type{}, s);
    }
    if (s == 3) {                                    // odd
        for (; s + 1 <= count - 3; s += 2) {
            step(Odd{}, std::false_type{}, s);
            step(Even{}, std::false_type{}, s + 1);
        }
    }
    for (; s <= count + 2; ++s) {
        if (s & 1) step(Odd{}, std::true_type{}, s);
        else step(Even{}, std::true_type{}, s);
    }
    __builtin_amdgcn_s_waitcnt(vmcnt_imm(0));        // nothing may still be on its way into LDS when the workgroup ends
}

// ------------------------------------------------------------------------------------------ host side
// Launch for one (H, P): picks the instantiation for the network's observation width and action count.
template <int H, int P, int OPS, bool QV>
hipError_t stream_launch_one(const ActStreamArgs &a, int groups, hipStream_t stream)
{
    // once per device: launches of this kernel may ask for more than 64 KB of dynamic LDS
    static std::atomic<uint64_t> allowed{0};
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return err;
    void (*kernel)(const ActStreamArgs) = act_stream_kernel<H, P, OPS, QV>;
    if (!(allowed.load(std::memory_order_acquire) & (1ull << (dev & 63)))) {
        err = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
        if (err != hipSuccess) return err;
        allowed.fetch_or(1ull << (dev & 63), std::memory_order_release);
    }
    const size_t lds_bytes = StreamLds<H, P>::total(a.net.D);
    launch_kernel(kernel, dim3((unsigned)groups), dim3(64 * (H / 16)), lds_bytes, stream, a);
    return hipGetLastError();
}

constexpr int kStreamMaxObsOps = 3;

template <int H, int P>
hipError_t stream_launch(const ActStreamArgs &a, int groups, hipStream_t stream)
{
    const int n_chunks = (64 * a.net.D + 1023) / 1024, ops = (n_chunks + H / 16 - 1) / (H / 16);
    const bool qv = (a.net.A & 3) == 0;
    switch (ops * 2 + (qv ? 1 : 0)) {
    case 2: return stream_launch_one<H, P, 1, false>(a, groups, stream);
    case 3: return stream_launch_one<H, P, 1, true>(a, groups, stream);
    case 4: return stream_launch_one<H, P, 2, false>(a, groups, stream);
    case 5: return stream_launch_one<H, P, 2, true>(a, groups, stream);
    case 6: return stream_launch_one<H, P, 3, false>(a, groups, stream);
    case 7: return stream_launch_one<H, P, 3, true>(a, groups, stream);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace marl
