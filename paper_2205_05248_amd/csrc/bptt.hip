// Backward half of the learner step for the recurrent Q-network: the gradient of
// sum(g * q_taken) with respect to every parameter, g = dL/dq_taken handed in by the caller.
//
//   unroll_fused_kernel<.., kTdSave>   (unroll_fused.hip) forward pass of the online network that keeps x and
//                                      h of every slot in global memory, [B, T+1, N, H]: h in fp32, x in fp32
//                                      or, for a bf16 network, in bf16 (what every reader rounds it to)
//   bptt_back_kernel                   one workgroup per 16 (episode, agent) rows walks the slots backwards.
//                                      Per slot it recomputes the gates from x_t and h_{t-1} (two MFMA
//                                      products, as the forward pass), forms the adjoints of the four gate
//                                      pre-activations, and carries dL/dh back through W_hh^T; W_ih^T gives
//                                      the adjoint of x and, through the ReLU, of fc1's pre-activation.  All
//                                      four GRU matrices stay on chip: W_hh, W_hh^T and W_ih^T as operand
//                                      fragments in registers (four waves, one per SIMD, up to 512 registers
//                                      each), W_ih in LDS.  The adjoints go to global memory.
//   tn_gemm_kernel                     the weight gradients are sums over all (row, slot) samples of outer
//                                      products adjoint x activation: C[p][q] = sum_m A[m][p] B[m][q], four
//                                      times (W_ih, W_hh, W1, W2).  The samples are split into chunks, one
//                                      workgroup each, which computes the whole (small) result for its chunk:
//                                      it stages 32 samples at a time through LDS (the contraction index has
//                                      to become the fragments' k), every element read from memory once, and
//                                      writes its partial sum; extra columns of B made up on the fly (a column
//                                      of ones, or the one-hot agent id) yield the bias gradients in the same
//                                      product.
//   tn_gemm_wide_kernel                the same products for a bf16 network: both operands are fetched 16 bytes
//                                      at a time and staged as they lie in memory; the transposing LDS read
//                                      turns the staged rows into fragments.
//   tn_reduce_kernel                   adds the chunks' partial sums in a fixed order and writes the result
//                                      into the packed gradient vector.
// A batch with fewer row tiles than compute units leaves most of the chip idle while bptt_back_kernel walks the
// slots.  For a bf16 network the slots are therefore walked in two launches (dL/dh handed over in memory), and the
// products over the later half run on a second stream of the handle's beside the earlier half's recurrence
// (launch_qnet_grad); the sum over all chunks, later half first, follows on the caller's stream.
// The precision follows the network's, in every product of the pass: fp32 networks split every operand into two
// bf16 planes (three MFMAs per product), bf16 networks round the operands (adjoints, activations) to bf16.
#include <type_traits>
#include <hip/hip_runtime.h>

#include <algorithm>

#include "fused16_roles.h"

namespace marl {

struct BpttArgs {
    NetFrags net;
    int B, T, a16;
    const int32_t *actions;      // [B, T, N]
    const uint8_t *filled;       // [B, T]
    const float *grad_q;         // [B, T, N]   dL/dq_taken
    const float *h_all;          // [B, T+1, N, H]   h_all[b, s] = state before slot s
    const void *x_all;           // [B, T+1, N, H]   x of slot s; fp32, or bf16 for a one-plane network
    // The adjoints, fp32 for fp32 networks and bf16 for bf16 networks (whose products round them to bf16 anyway:
    // stored rounded, they cost half the traffic to write here and to read in the weight-gradient products)
    void *da;                    // [B, T, N, 4H]   adjoints of the gate pre-activations: n (input side), r, z, n (hidden side)
    void *dpre1;                 // [B, T, N, H]    adjoint of fc1's pre-activation
    void *dq;                    // [B, T, N, a16]  adjoint of Q, dense (one non-zero per row)
    // The launch walks slots t_end - 1 .. t_begin.  One launch takes all of them (0, T); two take the later and
    // then the earlier slots and hand dL/dh over in `carry` [rows rounded up to 16][H] fp32, so that the later
    // slots' weight-gradient products can run beside the second launch.
    int t_begin, t_end;
    float *carry;
};

template <int H, int P> struct BpttShape {
    using Sh = Fused16<H, P>;
    static constexpr int KS = Sh::KS, FBK = Sh::FBK, NBC = Sh::NBC;
    // LDS: W_ih, one buffer of h and x fragments and the gate biases where the forward kernel has them;
    // the adjoint fragments (r, z, n: 3 KS k-steps; n hidden side: KS) where it keeps the observations
    static constexpr int oDa = Sh::oObs, oDhn = oDa + 3 * KS * Sh::kFrag, kBytes = oDhn + KS * Sh::kFrag;
};

// The wave's blocks of 16 units as operand fragments in LDS: two adjacent blocks make one k-step.  A wave with
// two blocks writes a whole fragment, a wave with one block its half of every lane's 16 bytes.
template <int P, int NBC>
__device__ __forceinline__ void publish_blocks(bf16x8 (*dst)[P][64], int w, int lane, const f32x4 (&v)[NBC])
{
    if constexpr (NBC == 2) {
        const Frag<P> f = frag_of_pair<P>(v[0], v[1]);
        dst[w][0][lane] = f.hi;
        if constexpr (P == 2) dst[w][1][lane] = f.lo;
    } else {
        typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
        bf16x4 hi, lo;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            hi[r] = (__bf16)v[0][r];
            lo[r] = (__bf16)(v[0][r] - (float)hi[r]);
        }
        char *at = reinterpret_cast<char *>(&dst[w / 2][0][lane]) + (w & 1) * 8;
        *reinterpret_cast<bf16x4 *>(at) = hi;
        if constexpr (P == 2) *reinterpret_cast<bf16x4 *>(at + 1024) = lo;
    }
}

// NW waves share the H / 16 blocks of hidden units: four waves (one per SIMD, up to 512 registers) or eight
// (two per SIMD, one block each, so that one wave's waits are another's work).
template <int H, int P, int NW>
__global__ __launch_bounds__(64 * NW, NW / 4) void bptt_back_kernel(BpttArgs a)
{
    using Sh = Fused16<H, P>;
    using Bs = BpttShape<H, P>;
    constexpr int KS = Sh::KS, FBK = Sh::FBK, NBC = FBK / NW;
    static_assert(NBC == 1 || NBC == 2, "one or two blocks of hidden units per wave");
    extern __shared__ __attribute__((aligned(16))) char lds[];
    typedef bf16x8 (*FragBuf)[P][64];
    const FragBuf hf = reinterpret_cast<FragBuf>(lds + Sh::oH), xf = reinterpret_cast<FragBuf>(lds + Sh::oX);
    const FragBuf daf = reinterpret_cast<FragBuf>(lds + Bs::oDa), dhf = reinterpret_cast<FragBuf>(lds + Bs::oDhn);
    bf16x8 *const wih_lds = reinterpret_cast<bf16x8 *>(lds + Sh::oWih);
    const float *gb = reinterpret_cast<const float *>(lds + Sh::oGBias);

    const NetFrags &net = a.net;
    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int N = net.N, A = net.A, T = a.T, S = T + 1;
    const int rows = a.B * N;
    const int row = blockIdx.x * 16 + c;
    const bool valid = row < rows;
    const int b = valid ? row / N : 0, n = valid ? row % N : 0;

    {
        constexpr int kVecs = 3 * FBK * KS * P * 64;
        for (int i = threadIdx.x; i < kVecs; i += 64 * NW) wih_lds[i] = net.wih_16[i];
    }
    if (w == 0) GruWave<H, P>::stage_gate_biases(lds, net, lane);

    // this wave's hidden units: blocks NBC w + j; forward W_hh rows of the three gates, and the rows of
    // W_hh^T and W_ih^T that produce its units of dL/dh and dL/dx
    WFrag<P> whh[3][NBC][KS], whhT[NBC][3 * KS], wihT[NBC][3 * KS];
    f32x4 bias_hn[NBC];
#pragma unroll
    for (int j = 0; j < NBC; ++j) {
        const int blk = NBC * w + j;
#pragma unroll
        for (int gate = 0; gate < 3; ++gate)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                whh[gate][j][ks] = load_wfrag<P>(net.whh_16 + ((size_t)((gate * FBK + blk) * KS + ks) * P) * 64 + lane);
#pragma unroll
        for (int ks = 0; ks < 3 * KS; ++ks) {
            whhT[j][ks] = load_wfrag<P>(net.whhT_16 + ((size_t)(blk * 3 * KS + ks) * P) * 64 + lane);
            wihT[j][ks] = load_wfrag<P>(net.wihT_16 + ((size_t)(blk * 3 * KS + ks) * P) * 64 + lane);
        }
        bias_hn[j] = load_feature4(net.bias_hn, blk, q4);
    }

    const int unit0 = 16 * NBC * w + 4 * q4;                       // + 16 j: the lane's four units of block j
    const size_t slot_stride = (size_t)N * H;
    const float *h_row = a.h_all + ((size_t)b * S * N + n) * H + unit0;
    constexpr int kBytesX = P == 1 ? 2 : 4;
    const char *x_row = static_cast<const char *>(a.x_all) + (((size_t)b * S * N + n) * H + unit0) * kBytesX;

    // The inputs of a slot are asked for one iteration before it; the chosen action, whose row of W2 is one
    // of those inputs, one iteration earlier still.  Nothing here is conditional (rows past the end read row 0).
    struct StepIn { f32x4 hp[NBC], xv[NBC], w2[NBC]; float gq_raw; uint8_t fil; int u; };
    auto load_action = [&](int t) { return a.actions[((size_t)b * T + t) * N + n]; };
    auto fetch = [&](int t, int u_raw) {
        StepIn in;
        const size_t bt = (size_t)b * T + t;
        in.u = min(max(u_raw, 0), A - 1);
        in.fil = a.filled[bt];
        in.gq_raw = a.grad_q[bt * N + n];
#pragma unroll
        for (int j = 0; j < NBC; ++j) {
            in.hp[j] = *reinterpret_cast<const f32x4 *>(h_row + (size_t)t * slot_stride + 16 * j);
            const char *xp = x_row + ((size_t)t * slot_stride + 16 * j) * kBytesX;
            if constexpr (P == 1) {      // four bf16 values, widened (bf16 is the upper half of an fp32)
                const uint2 raw = *reinterpret_cast<const uint2 *>(xp);
                in.xv[j][0] = __uint_as_float(raw.x << 16); in.xv[j][1] = __uint_as_float(raw.x & 0xFFFF0000u);
                in.xv[j][2] = __uint_as_float(raw.y << 16); in.xv[j][3] = __uint_as_float(raw.y & 0xFFFF0000u);
            } else {
                in.xv[j] = *reinterpret_cast<const f32x4 *>(xp);
            }
            in.w2[j] = *reinterpret_cast<const f32x4 *>(net.w2_plain + (size_t)in.u * H + unit0 + 16 * j);
        }
        return in;
    };

    f32x4 dh[NBC];                                                 // dL/dh flowing into the state after slot t
    float *const carry_row = a.carry + (size_t)(blockIdx.x * 16 + c) * H + unit0;      // rows past the end have room too
#pragma unroll
    for (int j = 0; j < NBC; ++j) {
#pragma unroll
        for (int r = 0; r < 4; ++r) dh[j][r] = 0.0f;
        if (a.t_end < T) dh[j] = *reinterpret_cast<const f32x4 *>(carry_row + 16 * j);
    }

    // Every global access inside the loop is unconditional, so that the loop body is straight-line code and
    // the waits for the prefetched inputs count exactly the stores issued after them: rows past the end
    // store through buffer descriptors at an offset beyond the descriptor, which the hardware drops.
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    constexpr uint32_t kDrop = 0xFFFFFFF0u;
    const size_t samples = (size_t)rows * T;
    constexpr uint32_t kElem = P == 1 ? 2u : 4u;                   // bytes per stored adjoint
    const __amdgpu_buffer_rsrc_t da_buf = __builtin_amdgcn_make_buffer_rsrc(a.da, 0, (int)(uint32_t)(samples * 4 * H * kElem), kRawBuffer);
    const __amdgpu_buffer_rsrc_t pre_buf = __builtin_amdgcn_make_buffer_rsrc(a.dpre1, 0, (int)(uint32_t)(samples * H * kElem), kRawBuffer);
    const __amdgpu_buffer_rsrc_t dq_buf = __builtin_amdgcn_make_buffer_rsrc(a.dq, 0, (int)(uint32_t)(samples * a.a16 * kElem), kRawBuffer);
    // four adjoints of one lane -> element offset `at` of the array behind `buf` (dropped for rows past the end)
    auto store4 = [&](const f32x4 &v, const __amdgpu_buffer_rsrc_t &buf, uint32_t at, uint32_t drop_mask) {
        if constexpr (P == 1) {
            typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
            typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
            bf16x4 r;
#pragma unroll
            for (int i = 0; i < 4; ++i) r[i] = (__bf16)v[i];
            __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, r), buf, (at * 2u) | drop_mask, 0, 0);
        } else {
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, v), buf, (at * 4u) | drop_mask, 0, 0);
        }
    };
    uint32_t drop = valid ? 0u : kDrop;
    asm volatile("" : "+v"(drop));
    const uint32_t drop_dq = (16 * w < a.a16) ? drop : kDrop;      // wave w writes block w of the row's dQ

    StepIn nxt = fetch(a.t_end - 1, load_action(a.t_end - 1));
    int u_ahead = load_action(max(a.t_end - 2, 0));
    // Nothing may be in flight when the loop is entered: the waits inside it are then the ones of the loop
    // itself (the entry would otherwise add its own, stricter ones, which make every iteration wait for the
    // previous iteration's stores).
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int j = 0; j < NBC; ++j) asm volatile("" : "+v"(nxt.hp[j]), "+v"(nxt.xv[j]), "+v"(nxt.w2[j]));
    asm volatile("" : "+v"(nxt.gq_raw), "+v"(u_ahead));
    lds_barrier();                                                 // W_ih and the biases are in LDS
    for (int t = a.t_end - 1; t >= a.t_begin; --t) {
        const StepIn in = nxt;
        const int u_next = u_ahead;
        u_ahead = load_action(max(t - 2, 0));
        nxt = fetch(max(t - 1, 0), u_next);
        const float gq = (valid && in.fil) ? in.gq_raw : 0.0f;
        publish_blocks<P, NBC>(hf, w, lane, in.hp);
        publish_blocks<P, NBC>(xf, w, lane, in.xv);
        lds_barrier();

        // the gates of slot t again
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
            Frag<P> hb, xb;
            hb.hi = hf[ks][0][lane];
            xb.hi = xf[ks][0][lane];
            if constexpr (P == 2) { hb.lo = hf[ks][1][lane]; xb.lo = xf[ks][1][lane]; }
#pragma unroll
            for (int j = 0; j < NBC; ++j) {
                const int blk = NBC * w + j;
                mma16<P>(acc_r[j], whh[0][j][ks], hb);
                mma16<P>(acc_z[j], whh[1][j][ks], hb);
                mma16<P>(acc_hn[j], whh[2][j][ks], hb);
                mma16<P>(acc_r[j], load_wfrag<P>(wih_lds + ((size_t)((0 * FBK + blk) * KS + ks) * P) * 64 + lane), xb);
                mma16<P>(acc_z[j], load_wfrag<P>(wih_lds + ((size_t)((1 * FBK + blk) * KS + ks) * P) * 64 + lane), xb);
                mma16<P>(acc_in[j], load_wfrag<P>(wih_lds + ((size_t)((2 * FBK + blk) * KS + ks) * P) * 64 + lane), xb);
            }
        }

        // adjoints of the pre-activations
        f32x4 dar[NBC], daz[NBC], dan[NBC], dahn[NBC], carry[NBC];
#pragma unroll
        for (int j = 0; j < NBC; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const float rr = sigmoidf_fast(acc_r[j][r]), zz = sigmoidf_fast(acc_z[j][r]);
                const float nn = tanhf_fast(acc_in[j][r] + rr * acc_hn[j][r]);
                const float dht = dh[j][r] + gq * in.w2[j][r];             // Q_t[u] = W2[u] . h_t + b2[u]
                const float dn = dht * (1.0f - zz) * (1.0f - nn * nn);
                dan[j][r] = dn;
                dahn[j][r] = dn * rr;
                dar[j][r] = dn * acc_hn[j][r] * rr * (1.0f - rr);
                daz[j][r] = dht * (in.hp[j][r] - nn) * zz * (1.0f - zz);
                carry[j][r] = dht * zz;
            }
        const uint32_t m = (uint32_t)((b * T + t) * N + n);          // sample index; the host bounds 4 H samples to 2^30
        {
            const uint32_t da_at = m * 4 * H + unit0;
#pragma unroll
            for (int j = 0; j < NBC; ++j) {
                store4(dan[j], da_buf, da_at + 0 * H + 16 * j, drop);
                store4(dar[j], da_buf, da_at + 1 * H + 16 * j, drop);
                store4(daz[j], da_buf, da_at + 2 * H + 16 * j, drop);
                store4(dahn[j], da_buf, da_at + 3 * H + 16 * j, drop);
            }
            // the adjoint of Q_t, dense: wave w writes action block w of every row
            f32x4 v;
#pragma unroll
            for (int r = 0; r < 4; ++r) v[r] = (16 * w + 4 * q4 + r == in.u) ? gq : 0.0f;
            store4(v, dq_buf, m * a.a16 + 16 * w + 4 * q4, drop_dq);
        }
        publish_blocks<P, NBC>(daf + 0 * KS, w, lane, dar);
        publish_blocks<P, NBC>(daf + 1 * KS, w, lane, daz);
        publish_blocks<P, NBC>(daf + 2 * KS, w, lane, dan);
        publish_blocks<P, NBC>(dhf, w, lane, dahn);
        lds_barrier();

        // back through the two products: dL/dh_{t-1} and dL/dx_t for this wave's units
        f32x4 accx[NBC];
#pragma unroll
        for (int j = 0; j < NBC; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) accx[j][r] = 0.0f;
#pragma unroll
        for (int ks = 0; ks < 3 * KS; ++ks) {
            Frag<P> di, dhid;
            di.hi = daf[ks][0][lane];
            if constexpr (P == 2) di.lo = daf[ks][1][lane];
            if (ks < 2 * KS) {
                dhid = di;
            } else {
                dhid.hi = dhf[ks - 2 * KS][0][lane];
                if constexpr (P == 2) dhid.lo = dhf[ks - 2 * KS][1][lane];
            }
#pragma unroll
            for (int j = 0; j < NBC; ++j) {
                mma16<P>(carry[j], whhT[j][ks], dhid);
                mma16<P>(accx[j], wihT[j][ks], di);
            }
        }
#pragma unroll
        for (int j = 0; j < NBC; ++j) {
            dh[j] = carry[j];
            f32x4 dp;
#pragma unroll
            for (int r = 0; r < 4; ++r) dp[r] = in.xv[j][r] > 0.0f ? accx[j][r] : 0.0f;
            store4(dp, pre_buf, m * H + unit0 + 16 * j, drop);
        }
    }
    if (a.t_begin > 0) {
#pragma unroll
        for (int j = 0; j < NBC; ++j) *reinterpret_cast<f32x4 *>(carry_row + 16 * j) = dh[j];
    }
}

// ------------------------------------------------------------------------------------------ weight gradients
struct TnGemmArgs {
    RowMap a, b;
    int M;              // samples
    int P, Q;           // columns of A and of B taken
    int extra_mode;     // columns appended to B: kExtraOnes (one column of ones), kExtraAgent (N one-hot columns of m % N)
    int n_extra, N;
    int qp;             // Q + n_extra rounded up to 16: row pitch of the result
    int chunk;          // samples per workgroup along the contraction, a multiple of 32
    // elements from a row to the next: inside a group, and from a group's last row to the next group's first
    // (A's rows are one group: the adjoint arrays are)
    unsigned next_a, next_b, wrap_b;
    unsigned wrap_a;    // tn_gemm_wide_kernel only: A in groups too
    float *partial;     // [chunks][128 or 384 rows][qp]
};

constexpr int kTnThreads = 512;        // eight waves: two per SIMD
constexpr int kTnBatchMax = 16;        // products of one shape launched together (blockIdx.y picks one)
struct TnGemmBatch { TnGemmArgs g[kTnBatchMax]; };

// One workgroup per chunk of samples computes the whole result, so that every operand element is read from
// memory once.  Wave w owns result row blocks w, w + 8, .. (PBW of them) and all QBN column blocks.  P: bf16
// planes per operand, the network's own: 2 = every value as bf16 high part + bf16 of the remainder, three MFMAs
// per product; 1 = values rounded to bf16, one MFMA.
// ABF: A's elements are bf16 (the adjoints of a bf16 network), else fp32.  BBF: the same for B's (its saved x).
template <int PBW, int QBN, int P, bool ABF, bool BBF = false>
__global__ __launch_bounds__(kTnThreads, 2) void tn_gemm_kernel(const TnGemmBatch batch)
{
    const TnGemmArgs g = batch.g[blockIdx.y];
    constexpr int kPp = 16 * 8 * PBW;                              // result rows, padded = columns of A staged
    constexpr int kSets = (kPp + 16 * QBN + 63) / 64;              // sets of 64 staged columns (A's, then B's)
    constexpr int kSetsPerWave = (kSets + 1) / 2;
    constexpr bool kTwoBuffers = P == 1;                           // a second staging buffer where it fits
    constexpr int kPitch = 80;                                     // bytes per column: 64 + 16 against bank conflicts
    // LDS: P planes (bf16 high part, bf16 of the remainder), each column-major: column c of the staged 32
    // samples is 64 bytes, the lane's eight samples of a fragment 16.
    extern __shared__ __attribute__((aligned(16))) char stage[];
    const int cols = kPp + g.qp;
    const int plane_bytes = cols * kPitch;
    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int sg = w & 3, half = w >> 2;                           // the wave stages samples 8 sg + 0..7 of every other column set
    const int n_qb = g.qp / 16;
    const int m_begin = (int)blockIdx.x * g.chunk, m_end = min(g.M, m_begin + g.chunk);     // M < 2^30
    // The 32 samples of a step are eight consecutive ones from each quarter of the chunk: wave group sg walks
    // through its own quarter, so that the rows it reads follow one another from the first step to the last and
    // their addresses are stepped, never recomputed.
    const int n_steps = (m_end - m_begin + 31) / 32;
    const int wave_begin = m_begin + 8 * n_steps * sg, wave_end = min(m_end, wave_begin + 8 * n_steps);

    f32x4 acc[PBW][QBN];
#pragma unroll
    for (int k = 0; k < PBW; ++k)
#pragma unroll
        for (int j = 0; j < QBN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[k][j][r] = 0.0f;

    // Inputs are asked for kDepth steps before they are used, into kDepth register sets that the unrolled
    // loop addresses statically.  Every load is unconditional (rows past the end of the arrays repeat the last
    // row, columns past an operand's width repeat its first), so the loop is straight-line code.
    constexpr int kDepth = 2;
    // bf16 adjoints (ABF) are not fetched column by column like the rest: a thread takes 16 bytes, eight columns
    // of one sample, and the tile goes to LDS as it lies in memory, sample-major; the transposition into
    // fragments (eight samples of one column per lane) is left to the transposing LDS read.  kAVec such loads
    // per thread cover the step's 32 samples of kPp columns.
    constexpr int kAVec = ABF ? 32 * kPp * 2 / 16 / kTnThreads : 0;
    constexpr int kAChunks = kPp / 8;                              // 16-byte pieces of a staged row of A
    constexpr int kAPitch = kPp * 2 + 32;                          // bytes from a sample's row to the next in LDS
    static_assert(!ABF || (32 * kPp * 2) % (16 * kTnThreads) == 0, "whole loads per thread");
    static_assert(32 * kAPitch <= kPp * kPitch, "the sample-major tile fits where A's columns would lie");
    struct Staged { float col[kSetsPerWave][8]; uint4 a[kAVec > 0 ? kAVec : 1]; };
    Staged rv[kDepth];
    // kPp is a multiple of 128, so set i of either half of the waves is one of A's exactly for i < kPp / 128:
    // known at compile time, and with it the element type, so that a load is one instruction with no branch
    constexpr int kSetsOfA = kPp / 128;
    static_assert(kPp % 128 == 0, "the column sets of A split evenly between the two halves of the waves");
    // Per column set of this wave: the lane's (clamped) column in its operand's rows, and for B's sets what the lane's
    // column is made of: -2 a column of B itself (or one past everything, whose results nobody reads), -1 the
    // appended column of ones, n >= 0 the appended one-hot column of agent n.
    int set_col[kSetsPerWave], made_of[kSetsPerWave];
#pragma unroll
    for (int i = 0; i < kSetsPerWave; ++i) {
        const int col = lane + 64 * (2 * i + half), cb = col - kPp;
        set_col[i] = i < kSetsOfA ? (col < g.P ? col : 0) : (cb < g.Q ? cb : 0);
        made_of[i] = (i >= kSetsOfA && cb >= g.Q && cb < g.Q + g.n_extra) ? (g.extra_mode == kExtraOnes ? -1 : cb - g.Q) : -2;
    }
    // A column past an operand's width is staged with the values of the operand's first column: it only reaches
    // rows or columns of the result that the reduction never reads, and costs no instruction here.

    // The row the next load takes, as addresses in A and B; (group, row in group) by division once, then by
    // stepping: a row further in the group, or from a group's last row to the next group's first.  All of it
    // is the same in every lane and is kept in scalar registers (said so where the compiler cannot tell).
    const unsigned row0 = (unsigned)min(wave_begin, g.M - 1);
    const unsigned gb0 = __builtin_amdgcn_readfirstlane(row0 / (unsigned)g.b.rows_per_group);
    const unsigned ib0 = row0 - gb0 * (unsigned)g.b.rows_per_group;
    long off_a = (long)row0 * g.a.ld;                                        // in elements; A's rows follow one another
    long off_b = (long)gb0 * g.b.group_stride + (long)ib0 * g.b.ld;
    unsigned b_left = (unsigned)g.b.rows_per_group - ib0;            // rows to the end of B's group
    unsigned rows_left = (unsigned)(g.M - 1) - row0;                  // steps that stay inside the arrays
    int sample = wave_begin;                                          // first sample of the step being staged
    unsigned agent0 = (unsigned)wave_begin % (unsigned)g.N;          // its agent, where rows are (.., agent) samples
    const unsigned agent_step = 8u % (unsigned)g.N;
    // wide loads of A: load i of this thread is piece a_piece of row a_k (sample 8 (a_k / 8) + a_k % 8 of the step:
    // the a_k % 8-th of quarter a_k / 8), at a_at bytes from A's base; every step moves eight rows on
    // (a_fetch: the sample the next load takes, a_staged: the one the next deposit puts down, a_end: the end of
    // the quarter's share)
    long a_at[kAVec > 0 ? kAVec : 1];
    int a_fetch[kAVec > 0 ? kAVec : 1], a_staged[kAVec > 0 ? kAVec : 1], a_end[kAVec > 0 ? kAVec : 1], a_lds[kAVec > 0 ? kAVec : 1];
    if constexpr (ABF) {
#pragma unroll
        for (int i = 0; i < kAVec; ++i) {
            const int v = (int)threadIdx.x + kTnThreads * i, k = v / kAChunks, piece = v % kAChunks;
            const int quarter_begin = m_begin + 8 * n_steps * (k >> 3);
            a_fetch[i] = a_staged[i] = quarter_begin + (k & 7);
            a_end[i] = min(m_end, quarter_begin + 8 * n_steps);
            a_at[i] = ((long)min(a_fetch[i], g.M - 1) * g.a.ld + (8 * piece < g.P ? 8 * piece : 0)) * 2;
            a_lds[i] = k * kAPitch + 16 * piece;
        }
    }

    // The loop comes twice.  ENDS = false: every row the workgroup touches, those fetched ahead included, exists
    // and every sample of every step counts - all chunks but the last one or two.  ENDS = true: past the last
    // sample the last row is fetched again (and not used), and samples past the wave's share are cleared (A's
    // values are; B's may stay).
    auto run = [&](auto ends_tag) {
        constexpr bool ENDS = decltype(ends_tag)::value;
        auto fetch = [&](Staged &into) {                             // this wave's next eight rows
            float (&f)[kSetsPerWave][8] = into.col;
            if constexpr (ABF) {
#pragma unroll
                for (int i = 0; i < kAVec; ++i) {
                    into.a[i] = *reinterpret_cast<const uint4 *>(static_cast<const char *>(g.a.base) + a_at[i]);
                    // eight rows on, or (ENDS) stay where the arrays end: what is fetched there again is not used
                    long step_bytes = (long)8 * g.next_a * 2;
                    if constexpr (ENDS) step_bytes = a_fetch[i] + 8 < g.M ? step_bytes : 0;
                    a_at[i] += step_bytes;
                    a_fetch[i] += 8;
                }
            }
#pragma unroll
            for (int r = 0; r < 8; ++r) {
                const char *arow = static_cast<const char *>(g.a.base) + off_a * (ABF ? 2 : 4);
                const char *brow = static_cast<const char *>(g.b.base) + off_b * (BBF ? 2 : 4);
#pragma unroll
                for (int i = ABF ? kSetsOfA : 0; i < kSetsPerWave; ++i) {
                    if constexpr (BBF) {
                        if (i >= kSetsOfA) {
                            f[i][r] = __uint_as_float((uint32_t)reinterpret_cast<const uint16_t *>(brow)[set_col[i]]);
                            continue;
                        }
                    }
                    f[i][r] = i < kSetsOfA ? reinterpret_cast<const float *>(arow)[set_col[i]] : reinterpret_cast<const float *>(brow)[set_col[i]];
                }
                // the next row, without a branch (a branch between two loads would make every wait a full one)
                unsigned go = 1u;
                if constexpr (ENDS) { go = rows_left ? 1u : 0u; rows_left -= go; }
                b_left -= go;
                const bool wb = b_left == 0u;
                unsigned sa = g.next_a, sb = wb ? g.wrap_b : g.next_b;      // A's rows are one group (the launcher checks)
                if constexpr (ENDS) { sa = go ? sa : 0u; sb = go ? sb : 0u; }
                off_a += sa; off_b += sb;
                asm volatile("" : "+s"(off_a));      // kept as one running scalar, not turned into a vector address per row
                b_left = wb ? (unsigned)g.b.rows_per_group : b_left;
            }
        };
        // The wave's eight samples of a column are samples 8 sg + 0..7 of the step: as bf16 they are exactly the
        // 16 bytes that lane quarter sg of a fragment of that column reads.  Converted once here, not by every
        // reader.  A loaded value is first passed through an empty asm: that is where the wait for it goes, and
        // it keeps the compiler from turning "loaded value or zero" into a branch around the load.
        auto deposit = [&](char *buf, Staged &from) {
            float (&f)[kSetsPerWave][8] = from.col;
            if constexpr (ABF) {
#pragma unroll
                for (int i = 0; i < kAVec; ++i) {
                    uint4 v = from.a[i];
                    asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
                    if constexpr (ENDS) {
                        const uint32_t keep = a_staged[i] < a_end[i] ? 0xFFFFFFFFu : 0u;
                        v.x &= keep; v.y &= keep; v.z &= keep; v.w &= keep;
                    }
                    *reinterpret_cast<uint4 *>(buf + a_lds[i]) = v;
                    a_staged[i] += 8;
                }
            }
#pragma unroll
            for (int i = ABF ? kSetsOfA : 0; i < kSetsPerWave; ++i) {
                const int col = lane + 64 * (2 * i + half);
                if constexpr (BBF) {
                    if (i >= kSetsOfA) {      // bf16 values of B, or the bf16 of an appended column's 1 or 0
                        uint32_t word[4];
                        unsigned agent = agent0;
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            asm volatile("" : "+v"(f[i][2 * j]), "+v"(f[i][2 * j + 1]));
                            uint32_t e[2];
#pragma unroll
                            for (int k = 0; k < 2; ++k) {
                                const int which = g.extra_mode == kExtraOnes ? -1 : (int)agent;
                                e[k] = made_of[i] == which ? 0x3F80u : (made_of[i] == -2 ? __float_as_uint(f[i][2 * j + k]) : 0u);
                                agent = agent + 1 == (unsigned)g.N ? 0u : agent + 1;
                            }
                            word[j] = e[0] | (e[1] << 16);
                        }
                        if (col < cols) *reinterpret_cast<uint4 *>(buf + col * kPitch + 16 * sg) = make_uint4(word[0], word[1], word[2], word[3]);
                        continue;
                    }
                }
                float v[8];
                unsigned agent = agent0;
#pragma unroll
                for (int r = 0; r < 8; ++r) {
                    asm volatile("" : "+v"(f[i][r]));
                    if (i < kSetsOfA) {
                        v[r] = (!ENDS || sample + r < wave_end) ? f[i][r] : 0.0f;
                    } else {
                        const int which = g.extra_mode == kExtraOnes ? -1 : (int)agent;
                        v[r] = made_of[i] == which ? 1.0f : (made_of[i] == -2 ? f[i][r] : 0.0f);
                        agent = agent + 1 == (unsigned)g.N ? 0u : agent + 1;
                    }
                }
                if (col < cols) {
                    const Frag<P> fr = to_frag<P>(v);
                    *reinterpret_cast<bf16x8 *>(buf + col * kPitch + 16 * sg) = fr.hi;
                    if constexpr (P == 2) *reinterpret_cast<bf16x8 *>(buf + plane_bytes + col * kPitch + 16 * sg) = fr.lo;
                }
            }
            sample += 8;
            agent0 += agent_step;
            agent0 = agent0 >= (unsigned)g.N ? agent0 - (unsigned)g.N : agent0;
        };

#pragma unroll
        for (int d = 0; d < kDepth; ++d) fetch(rv[d]);
        // fragments: lane (c, q4) takes samples 8 q4 + 0..7 of column 16 block + c
        auto multiply = [&](const char *buf) {
            const char *mine = buf + c * kPitch + 16 * q4;
            WFrag<P> af[PBW];
#pragma unroll
            for (int k = 0; k < PBW; ++k) {
                if constexpr (ABF) {
                    // The transposing read works on blocks of 16 lanes: lane 4 a + e of a block receives, as its
                    // i-th value, element e of the four that lane a + 4 i of the block points at.  With lane a + 4 i
                    // pointing at sample 8 q4 + i, columns 4 a .. 4 a + 3, lane c gets column c of samples
                    // 8 q4 + 0..3; the second read gives samples 8 q4 + 4..7.
                    typedef short s16x4 __attribute__((ext_vector_type(4)));
                    typedef s16x4 __attribute__((address_space(3))) *LdsQuad;
                    const char *at = buf + (8 * q4 + (c >> 2)) * kAPitch + (16 * (w + 8 * k) + 4 * (c & 3)) * 2;
                    const s16x4 first = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LdsQuad)(at));
                    const s16x4 second = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LdsQuad)(at + 4 * kAPitch));
                    typedef short s16x8 __attribute__((ext_vector_type(8)));
                    const s16x8 both = __builtin_shufflevector(first, second, 0, 1, 2, 3, 4, 5, 6, 7);
                    af[k].hi = __builtin_bit_cast(bf16x8, both);
                } else {
                    af[k].hi = *reinterpret_cast<const bf16x8 *>(mine + 16 * (w + 8 * k) * kPitch);
                    if constexpr (P == 2) af[k].lo = *reinterpret_cast<const bf16x8 *>(mine + plane_bytes + 16 * (w + 8 * k) * kPitch);
                }
            }
#pragma unroll
            for (int j = 0; j < QBN; ++j)
                if (j < n_qb) {
                    Frag<P> bf;
                    bf.hi = *reinterpret_cast<const bf16x8 *>(mine + (kPp + 16 * j) * kPitch);
                    if constexpr (P == 2) bf.lo = *reinterpret_cast<const bf16x8 *>(mine + plane_bytes + (kPp + 16 * j) * kPitch);
#pragma unroll
                    for (int k = 0; k < PBW; ++k) mma16<P>(acc[k][j], af[k], bf);
                }
        };
        // Rounds of kDepth steps; steps past the end of the chunk add zeros.  The compiler's wait at the head of
        // the loop is for everything asked for so far, whatever the order of the round.  Where two staging
        // buffers fit, the round is therefore: stage both steps, ask for the next two, multiply both - every
        // load has both multiplications to arrive in.
        for (int s0 = 0; s0 < n_steps; s0 += kDepth) {
            if constexpr (kTwoBuffers) {
                static_assert(kDepth == 2, "one staging buffer per step of a round");
                char *second = stage + P * plane_bytes;
                deposit(stage, rv[0]);
                deposit(second, rv[1]);
                fetch(rv[0]);
                fetch(rv[1]);
                __syncthreads();
                multiply(stage);
                multiply(second);
                __syncthreads();               // every wave is done reading before the next round writes
            } else {
#pragma unroll
                for (int d = 0; d < kDepth; ++d) {
                    __syncthreads();           // one buffer: the previous step has been read by every wave
                    deposit(stage, rv[d]);
                    fetch(rv[d]);              // asked for before the barrier, so that the wait at it is not idle time for memory
                    __syncthreads();
                    multiply(stage);
                }
            }
        }
    };
    // Rows touched: the last quarter's, plus what is fetched ahead of the last step (the loop runs whole rounds).
    const int rounds_end = (n_steps + kDepth - 1) / kDepth * kDepth;
    const bool all_inside = m_begin + 8 * (3 * n_steps + rounds_end + kDepth) <= g.M
                            && rounds_end == n_steps && m_end - m_begin == 32 * n_steps;
    // (two planes: the one general loop only - twice over, the loop did not fit the registers)
    if (P == 1 && all_inside) run(std::integral_constant<bool, P != 1>{});
    else run(std::true_type{});

    // C layout: lane (c, q4) holds result[16 block + 4 q4 + r][16 j + c]
    float *out = g.partial + (size_t)blockIdx.x * kPp * g.qp;
#pragma unroll
    for (int k = 0; k < PBW; ++k)
#pragma unroll
        for (int j = 0; j < QBN; ++j)
            if (j < n_qb)
#pragma unroll
                for (int r = 0; r < 4; ++r) out[(size_t)(16 * (w + 8 * k) + 4 * q4 + r) * g.qp + 16 * j + c] = acc[k][j][r];
}

// The same product for a bf16 network whose operands allow it (tn_wide_fits): neither operand is fetched
// column by column.  A thread takes 16 bytes of a sample's row (eight bf16 or four fp32 columns), the step's 32
// samples go to LDS as they lie in memory, sample-major and as bf16, and the transposition into fragments
// (eight samples of one column per lane) is left to the transposing LDS read: a tenth of the load
// instructions.  Chunks, the order of samples within a step (eight consecutive ones from each quarter of the
// chunk), the made-up columns and the partial results are those of tn_gemm_kernel.
template <int PBW, int QBN, bool BBF>
__global__ __launch_bounds__(kTnThreads, 2) void tn_gemm_wide_kernel(const TnGemmBatch batch)
{
    const TnGemmArgs g = batch.g[blockIdx.y];
    constexpr int kPp = 16 * 8 * PBW;                              // result rows, padded = columns of A staged
    constexpr int kQp = 16 * QBN;                                  // most columns of B staged
    constexpr int kColsB = BBF ? 8 : 4;                            // columns of B in 16 bytes
    static_assert(kPp / 8 % 16 == 0, "whole loads of A per thread");
    // bytes from a sample's row to the next in LDS: 48 past a multiple of 256, so that the four rows a block of
    // 16 lanes reads together, 32 bytes of each, lie in different banks
    constexpr int kAPitch = kPp * 2 + 48, kBPitch = (kQp * 2 + 255) / 256 * 256 + 48;
    constexpr int kBufBytes = 32 * (kAPitch + kBPitch);
    extern __shared__ __attribute__((aligned(16))) char stage[];
    const int lane = threadIdx.x & 63, q4 = lane >> 4, c = lane & 15;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n_qb = g.qp / 16;
    const int m_begin = (int)blockIdx.x * g.chunk, m_end = min(g.M, m_begin + g.chunk);     // M < 2^30
    const int n_steps = (m_end - m_begin + 31) / 32;

    // Which blocks of the result a wave owns.  Three row blocks (w, w + 8, w + 16) and every column block where the
    // result is tall: a fragment of B then feeds three products.  Where it is 128 rows by up to 336 columns, all
    // eight row blocks and every eighth column block (w, w + 8, w + 16): 11 fragments per step for 24 products,
    // where one row block and all 21 column blocks would read 22 for 21 - and a wave can only issue so many LDS reads.
    constexpr bool kSplitColumns = PBW == 1;
    constexpr int kRB = kSplitColumns ? 8 : PBW, kCB = kSplitColumns ? (QBN + 7) / 8 : QBN;
    auto row_block = [&](int k) { return kSplitColumns ? k : w + 8 * k; };
    auto col_block = [&](int j) { return kSplitColumns ? w + 8 * j : j; };
    f32x4 acc[kRB][kCB];
#pragma unroll
    for (int k = 0; k < kRB; ++k)
#pragma unroll
        for (int j = 0; j < kCB; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) acc[k][j][r] = 0.0f;

    // A thread's loads all take pieces of one row: thread (quarter t / 128, row (t % 128) / 16, first piece t % 16)
    // fetches pieces first + 16 i of row 8 quarter + row of the step, i.e. of that quarter's next sample but
    // `row`, so that one address, one sample number and one end serve them all.  Pieces past the operand's
    // width repeat the first one (their results are rows or columns nobody reads, or they are made up below).
    constexpr int kALoads = kPp / 8 / 16;                          // per thread and step: of A,
    constexpr int kBLoads = (kQp / kColsB + 15) / 16;              // of B
    const int quarter = (int)threadIdx.x >> 7, row_in_quarter = ((int)threadIdx.x & 127) >> 4, first_piece = (int)threadIdx.x & 15;
    const int k_row = 8 * quarter + row_in_quarter;
    const int pieces_b = g.qp / kColsB;
    int sample_next = m_begin + 8 * n_steps * quarter + row_in_quarter;      // the sample the next loads take
    const int share_end = min(m_end, m_begin + 8 * n_steps * (quarter + 1));  // end of the quarter's share of the chunk
    const char *a_row, *b_row;                                     // the next loads' rows
    unsigned a_left, b_left;                                       // rows from the next load's to the end of its group
    unsigned agent;                                                // of the sample being staged next
    {
        const unsigned row = (unsigned)min(sample_next, g.M - 1);
        const unsigned group = row / (unsigned)g.b.rows_per_group, in_group = row - group * (unsigned)g.b.rows_per_group;
        const unsigned group_a = row / (unsigned)g.a.rows_per_group, in_group_a = row - group_a * (unsigned)g.a.rows_per_group;
        a_row = static_cast<const char *>(g.a.base) + ((long)group_a * g.a.group_stride + (long)in_group_a * g.a.ld) * 2;
        b_row = static_cast<const char *>(g.b.base) + ((long)group * g.b.group_stride + (long)in_group * g.b.ld) * (BBF ? 2 : 4);
        a_left = (unsigned)g.a.rows_per_group - in_group_a;
        b_left = (unsigned)g.b.rows_per_group - in_group;
        agent = (unsigned)sample_next % (unsigned)g.N;
    }
    const unsigned agent_step = 8u % (unsigned)g.N;
    int a_piece[kALoads], b_piece[kBLoads];                        // byte offsets within the row
#pragma unroll
    for (int i = 0; i < kALoads; ++i) a_piece[i] = 8 * (first_piece + 16 * i) < g.P ? 16 * (first_piece + 16 * i) : 0;
#pragma unroll
    for (int i = 0; i < kBLoads; ++i) b_piece[i] = kColsB * (first_piece + 16 * i) < g.Q ? 16 * (first_piece + 16 * i) : 0;
    const int a_lds = k_row * kAPitch + 16 * first_piece;          // + 256 i
    const int b_lds = 32 * kAPitch + k_row * kBPitch + 2 * kColsB * first_piece;      // + 32 kColsB i
    const int b_spare = 32 * kAPitch + k_row * kBPitch + (kBPitch - 48);             // 48 bytes that no fragment reads

    constexpr int kDepth = 2;
    struct Staged { uint4 a[kALoads], b[kBLoads]; };
    Staged rv[kDepth];
    int staged_sample = sample_next;                               // the sample the next deposit puts down

    auto run = [&](auto ends_tag) {
        constexpr bool ENDS = decltype(ends_tag)::value;           // the chunk reaches the end of the samples
        auto fetch = [&](Staged &into) {
#pragma unroll
            for (int i = 0; i < kALoads; ++i) into.a[i] = *reinterpret_cast<const uint4 *>(a_row + a_piece[i]);
#pragma unroll
            for (int i = 0; i < kBLoads; ++i) into.b[i] = *reinterpret_cast<const uint4 *>(b_row + b_piece[i]);
            // eight rows on: inside the group, or seven steps inside and one from a group's last row to the
            // next group's first.  (ENDS) Past the arrays' end the rows stay: what is fetched there again is not used.
            bool go = true;
            if constexpr (ENDS) go = sample_next + 8 < g.M;
            const bool wraps = b_left <= 8u, wraps_a = a_left <= 8u;
            const long b_step = (wraps ? (long)7 * g.next_b + g.wrap_b : (long)8 * g.next_b) * (BBF ? 2 : 4);
            const long a_step = (wraps_a ? (long)7 * g.next_a + g.wrap_a : (long)8 * g.next_a) * 2;
            a_row += go ? a_step : 0;
            b_row += go ? b_step : 0;
            a_left = go ? (wraps_a ? a_left + (unsigned)g.a.rows_per_group - 8u : a_left - 8u) : a_left;
            b_left = go ? (wraps ? b_left + (unsigned)g.b.rows_per_group - 8u : b_left - 8u) : b_left;
            sample_next += 8;
        };
        auto deposit = [&](char *buf, Staged &from) {
            uint32_t keep = 0xFFFFFFFFu;       // samples past the chunk's end count for nothing: A's values are cleared, B's may stay
            if constexpr (ENDS) keep = staged_sample < share_end ? 0xFFFFFFFFu : 0u;
#pragma unroll
            for (int i = 0; i < kALoads; ++i) {
                uint4 v = from.a[i];
                asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
                if constexpr (ENDS) { v.x &= keep; v.y &= keep; v.z &= keep; v.w &= keep; }
                *reinterpret_cast<uint4 *>(buf + a_lds + 256 * i) = v;
            }
#pragma unroll
            for (int i = 0; i < kBLoads; ++i) {
                uint4 v = from.b[i];
                asm volatile("" : "+v"(v.x), "+v"(v.y), "+v"(v.z), "+v"(v.w));
                const int piece = first_piece + 16 * i, col = kColsB * piece;
                // a piece past B's own columns is made up: the column of ones, or the one-hot columns of the sample's agent
                const bool made_up = col >= g.Q;
                uint32_t word[kColsB / 2];
#pragma unroll
                for (int e = 0; e < kColsB / 2; ++e) {
                    uint32_t pair[2];
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int extra = col + 2 * e + h - g.Q;            // which appended column, if any
                        const bool one = extra >= 0 && extra < g.n_extra && (g.extra_mode == kExtraOnes || (unsigned)extra == agent);
                        pair[h] = one ? 0x3F80u : 0u;
                    }
                    word[e] = pair[0] | (pair[1] << 16);
                }
                // a spare load (a piece past the staged columns) goes to the padding at the end of the row
                const int at = piece < pieces_b ? b_lds + 32 * kColsB * i : b_spare;
                if constexpr (BBF) {
                    const uint4 out = made_up && piece < pieces_b ? make_uint4(word[0], word[1], word[2], word[3]) : v;
                    *reinterpret_cast<uint4 *>(buf + at) = out;
                } else {
                    typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                    bf16x4 r;
                    r[0] = (__bf16)__uint_as_float(v.x); r[1] = (__bf16)__uint_as_float(v.y);
                    r[2] = (__bf16)__uint_as_float(v.z); r[3] = (__bf16)__uint_as_float(v.w);
                    const uint2 real = __builtin_bit_cast(uint2, r);
                    const uint2 out = made_up && piece < pieces_b ? make_uint2(word[0], word[1]) : real;
                    *reinterpret_cast<uint2 *>(buf + at) = out;
                }
            }
            staged_sample += 8;
            agent += agent_step;
            agent = agent >= (unsigned)g.N ? agent - (unsigned)g.N : agent;
        };
        // The transposing read works on blocks of 16 lanes: lane 4 a + e of a block receives, as its i-th value,
        // element e of the four that lane a + 4 i of the block points at.  With lane a + 4 i pointing at sample
        // 8 q4 + i, columns 4 a .. 4 a + 3 of a block of 16 columns, lane c gets column c of samples 8 q4 + 0..3;
        // a second read four rows on gives samples 8 q4 + 4..7: the fragment of lane (c, q4).
        auto fragment = [&](const char *rows, int pitch, int first_col) {
            typedef short s16x4 __attribute__((ext_vector_type(4)));
            typedef short s16x8 __attribute__((ext_vector_type(8)));
            typedef s16x4 __attribute__((address_space(3))) *LdsQuad;
            const char *at = rows + (8 * q4 + (c >> 2)) * pitch + (first_col + 4 * (c & 3)) * 2;
            const s16x4 first = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LdsQuad)(at));
            const s16x4 second = __builtin_amdgcn_ds_read_tr16_b64_v4i16((LdsQuad)(at + 4 * pitch));
            return __builtin_bit_cast(bf16x8, (s16x8)__builtin_shufflevector(first, second, 0, 1, 2, 3, 4, 5, 6, 7));
        };
        auto multiply = [&](const char *buf) {
            WFrag<1> af[kRB];
#pragma unroll
            for (int k = 0; k < kRB; ++k) af[k].hi = fragment(buf, kAPitch, 16 * row_block(k));
#pragma unroll
            for (int j = 0; j < kCB; ++j)
                if (col_block(j) < n_qb) {
                    Frag<1> bf;
                    bf.hi = fragment(buf + 32 * kAPitch, kBPitch, 16 * col_block(j));
#pragma unroll
                    for (int k = 0; k < kRB; ++k) mma16<1>(acc[k][j], af[k], bf);
                }
        };
#pragma unroll
        for (int d = 0; d < kDepth; ++d) fetch(rv[d]);
        // a round: stage both steps, ask for the next two, multiply both - every load has both multiplications to arrive in
        for (int s0 = 0; s0 < n_steps; s0 += kDepth) {
            deposit(stage, rv[0]);
            deposit(stage + kBufBytes, rv[1]);
            fetch(rv[0]);
            fetch(rv[1]);
            __syncthreads();
            multiply(stage);
            multiply(stage + kBufBytes);
            __syncthreads();                   // every wave is done reading before the next round writes
        }
    };
    // Rows touched: the last quarter's, plus what is fetched ahead of the last step (the loop runs whole rounds).
    const int rounds_end = (n_steps + kDepth - 1) / kDepth * kDepth;
    const bool all_inside = m_begin + 8 * (3 * n_steps + rounds_end + kDepth) <= g.M
                            && rounds_end == n_steps && m_end - m_begin == 32 * n_steps;
    if (all_inside) run(std::false_type{});
    else run(std::true_type{});

    // C layout: lane (c, q4) holds result[16 block + 4 q4 + r][16 j + c]
    float *out = g.partial + (size_t)blockIdx.x * kPp * g.qp;
#pragma unroll
    for (int k = 0; k < kRB; ++k)
#pragma unroll
        for (int j = 0; j < kCB; ++j)
            if (col_block(j) < n_qb)
#pragma unroll
                for (int r = 0; r < 4; ++r) out[(size_t)(16 * row_block(k) + 4 * q4 + r) * g.qp + 16 * col_block(j) + c] = acc[k][j][r];
}

template <int PBW, int QBN> constexpr size_t tn_wide_lds()
{
    return (size_t)2 * 32 * ((16 * 8 * PBW * 2 + 48) + ((16 * QBN * 2 + 255) / 256 * 256 + 48));
}

// Whether tn_gemm_wide_kernel can take a product: bf16 adjoints, and every row of both operands a whole number
// of 16-byte pieces at 16-byte aligned addresses, B's own columns ending on a piece.
bool tn_wide_fits(const TnProduct &t, long M)
{
    if (!t.a.bf16) return false;
    const int cols_b = t.b.bf16 ? 8 : 4, bytes_b = t.b.bf16 ? 2 : 4;
    if (reinterpret_cast<uintptr_t>(t.a.base) % 16 != 0 || t.a.ld % 8 != 0 || t.a.ld < (t.P + 7) / 8 * 8) return false;
    if (t.a.rows_per_group < M && (t.a.rows_per_group < 8 || (t.a.group_stride * 2) % 16 != 0)) return false;
    if (t.Q == 0) return t.b.ld >= cols_b && t.b.ld % cols_b == 0 && reinterpret_cast<uintptr_t>(t.b.base) % 16 == 0
                         && (t.b.rows_per_group >= M || (t.b.rows_per_group >= 8 && (t.b.group_stride * bytes_b) % 16 == 0));
    if (reinterpret_cast<uintptr_t>(t.b.base) % 16 != 0 || t.b.ld % cols_b != 0 || t.Q % cols_b != 0 || t.b.ld < cols_b) return false;
    if (t.b.rows_per_group < M && (t.b.rows_per_group < 8 || (t.b.group_stride * bytes_b) % 16 != 0)) return false;
    return true;
}

// Sum of the chunks, in a fixed order, into the packed gradient vector.  Result row p goes to row
// (p + row_shift) % P of the destination matrix (the adjoint array lists the gates as n, r, z, the
// parameters as r, z, n); columns < Q go to dst_w[row * ld_w + column]; the appended column of ones
// goes to dst_b[row]; appended agent columns continue the row of dst_w (they are W1's id columns).
struct TnReduceArgs {
    const float *partial;
    int chunks, P, p_pad, qp;
    int Q, n_extra, extra_mode;
    int row_shift, w_cols, ld_w;
    float *dst_w, *dst_b;
};
struct TnReduceBatch { TnReduceArgs r[kTnBatchMax]; };

__global__ void tn_reduce_kernel(const TnReduceBatch batch)
{
    const TnReduceArgs g = batch.r[blockIdx.y];
    const int cols = g.Q + g.n_extra;
    const int idx = blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= g.P * cols) return;
    const int p = idx / cols, q = idx % cols;
    const int row = (p + g.row_shift) % g.P;
    // four running sums over interleaved chunks keep sixteen loads in flight; the order is fixed
    const float *src = g.partial + (size_t)p * g.qp + q;
    const size_t step = (size_t)g.p_pad * g.qp;
    float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    int ch = 0;
    for (; ch + 16 <= g.chunks; ch += 16) {
        float v[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) v[i] = src[(size_t)(ch + i) * step];
#pragma unroll
        for (int i = 0; i < 16; ++i) s[i & 3] += v[i];
    }
    for (; ch < g.chunks; ++ch) s[ch & 3] += src[(size_t)ch * step];
    const float total = (s[0] + s[1]) + (s[2] + s[3]);
    if (q < g.Q || g.extra_mode == kExtraAgent) g.dst_w[(size_t)row * g.ld_w + q] = total;
    else g.dst_b[row] = total;
}

// kExtraAgent: the bias gradient is the sum of the agent columns just written.
__global__ void bias_from_columns_kernel(const float *w, int rows, int ld, int first, int count, float *dst)
{
    const int row = blockIdx.x * blockDim.x + threadIdx.x;
    if (row >= rows) return;
    float s = 0.0f;
    for (int e = 0; e < count; ++e) s += w[(size_t)row * ld + first + e];
    dst[row] = s;
}

// ------------------------------------------------------------------------------------------ host side
namespace {

size_t align_up(size_t v) { return (v + 255) / 256 * 256; }

struct Plan {
    size_t off_h, off_x, off_da, off_dpre1, off_dq, off_carry, off_partial, partial_bytes, bytes;
    int a16, chunks, chunk;
};

Plan make_plan(const NetFrags &net, int B, int T)
{
    Plan p{};
    const size_t adj = net.planes == 1 ? 2 : 4;                    // bytes per stored adjoint
    const size_t R = (size_t)B * net.N, S = (size_t)T + 1, H = net.H;
    p.a16 = (net.A + 15) / 16 * 16;
    const long M = (long)R * T;
    p.chunks = (int)std::min<long>(256, (M + 31) / 32);
    if (p.chunks < 1) p.chunks = 1;
    p.chunk = (int)(((M + p.chunks - 1) / p.chunks + 63) / 64 * 64);      // whole rounds of two steps of 32 samples
    size_t off = 0;
    p.off_h = off;      off = align_up(off + R * S * H * 4);
    p.off_x = off;      off = align_up(off + R * S * H * adj + 4);         // x: bf16 for a one-plane network
    p.off_da = off;     off = align_up(off + R * T * 4 * H * adj + 4);
    p.off_dpre1 = off;  off = align_up(off + R * T * H * adj + 4);
    p.off_dq = off;     off = align_up(off + R * T * p.a16 * adj + 4);
    // the four products run together: room for all their partial results
    const long chunks_real = (M + p.chunk - 1) / p.chunk;
    auto part = [&](size_t P, size_t Qt) { return (size_t)chunks_real * (P > 128 ? 384 : 128) * ((Qt + 15) / 16 * 16) * 4; };
    // (one-plane networks: twice, for the two halves of the slots whose products run apart, each in up to 256 chunks)
    const size_t need = (net.planes == 1 ? 2 : 1) * (2 * part(3 * H, H + 1) + part(H, (size_t)net.D + net.N) + part(net.A, H + 1));
    p.partial_bytes = need;
    p.off_carry = off;  off = align_up(off + (R + 15) / 16 * 16 * H * 4);
    p.off_partial = off; off = align_up(off + need);
    p.bytes = off;
    return p;
}

template <int H, int P, int NW>
hipError_t back_dispatch(const BpttArgs &a, hipStream_t stream)
{
    const int tiles = (a.B * a.net.N + 15) / 16;
    hipError_t err = allow_large_lds<bptt_back_kernel<H, P, NW>>(kLdsLimit);
    if (err != hipSuccess) return err;
    constexpr size_t kLds = BpttShape<H, P>::kBytes;
    hipLaunchKernelGGL((bptt_back_kernel<H, P, NW>), dim3(tiles), dim3(64 * NW), kLds, stream, a);
    return hipGetLastError();
}

}  // namespace

size_t tn_partial_bytes(long M, int chunk, int P, int q_total)
{
    const size_t chunks = (size_t)((M + chunk - 1) / chunk);
    return chunks * (P > 128 ? 384 : 128) * (size_t)((q_total + 15) / 16 * 16) * sizeof(float);
}

// Launches the products of `list` (all over the same M samples, chunks of `chunk`): those of one shape go
// together in one launch (up to kTnBatchMax), then their partial sums are reduced, again in one launch.
hipError_t launch_tn_products(int planes, const TnProduct *list, int count, long M, int chunk, float *partial,
                              size_t partial_bytes, hipStream_t stream)
{
    const int chunks = (int)((M + chunk - 1) / chunk);
    int done = 0;
    while (done < count) {
        TnGemmBatch wide{}, narrow{};
        TnReduceBatch red{};
        int n_wide = 0, n_narrow = 0, n_red = 0, max_q_wide = 0, max_q_narrow = 0, max_total = 0;
        size_t used = 0;
        int taken = done;
        bool a_in_groups = false;
        for (; taken < count; ++taken) {
            const TnProduct &t = list[taken];
            TnGemmArgs g{};
            g.a = t.a; g.b = t.b; g.M = (int)M; g.P = t.P; g.Q = t.Q; g.extra_mode = t.extra_mode; g.n_extra = t.n_extra;
            g.N = t.N > 0 ? t.N : 1;
            g.qp = (t.Q + t.n_extra + 15) / 16 * 16;
            g.chunk = chunk;
            // steps from row to row in elements, 32 bits each; an operand that is one group never takes the second
            auto steps = [&](const RowMap &m, unsigned *next, unsigned *wrap) {
                const long n = (long)m.ld;
                const long w = m.rows_per_group >= M ? n : m.group_stride - (long)(m.rows_per_group - 1) * m.ld;
                if (n < 0 || w < 0 || n >= (1L << 31) || w >= (1L << 31)) return false;
                *next = (unsigned)n; *wrap = (unsigned)w;
                return true;
            };
            if (!steps(t.a, &g.next_a, &g.wrap_a) || !steps(t.b, &g.next_b, &g.wrap_b)) return hipErrorInvalidValue;
            // A in groups: the wide kernel only
            if (t.a.rows_per_group < M && !(planes == 1 && tn_wide_fits(t, M))) return hipErrorInvalidValue;
            a_in_groups = a_in_groups || t.a.rows_per_group < M;
            // bf16 adjoints are read 16 bytes (eight columns) at a time
            if (t.a.bf16 && (reinterpret_cast<uintptr_t>(t.a.base) % 16 != 0 || t.a.ld % 8 != 0 || t.a.ld < (t.P + 7) / 8 * 8)) return hipErrorInvalidValue;
            // two shapes: up to 384 rows x 144 columns (the GRU matrices), up to 128 rows x 336 columns (fc1, fc2)
            const bool is_wide = t.P > 128;
            if ((is_wide && (t.P > 384 || g.qp > 144)) || (!is_wide && g.qp > 336)) return hipErrorInvalidValue;
            if ((t.a.bf16 != 0) != (list[0].a.bf16 != 0) || (t.a.bf16 && planes != 1)) return hipErrorInvalidValue;
            // B in bf16: the wide shape of a one-plane network with bf16 adjoints only; such products go in launches of their own
            if (t.b.bf16 && !(is_wide && t.a.bf16)) return hipErrorInvalidValue;
            if ((t.b.bf16 != 0) != (list[done].b.bf16 != 0)) break;
            const size_t bytes = tn_partial_bytes(M, chunk, t.P, t.Q + t.n_extra);
            if (bytes > partial_bytes) return hipErrorInvalidValue;
            if (used + bytes > partial_bytes || (is_wide ? n_wide : n_narrow) == kTnBatchMax || n_red == kTnBatchMax) break;
            g.partial = reinterpret_cast<float *>(reinterpret_cast<char *>(partial) + used);
            used += bytes;
            if (is_wide) { wide.g[n_wide++] = g; max_q_wide = std::max(max_q_wide, g.qp); }
            else         { narrow.g[n_narrow++] = g; max_q_narrow = std::max(max_q_narrow, g.qp); }
            TnReduceArgs r{};
            r.partial = g.partial; r.chunks = chunks; r.P = t.P; r.p_pad = is_wide ? 384 : 128; r.qp = g.qp;
            r.Q = t.Q; r.n_extra = t.n_extra; r.extra_mode = t.extra_mode;
            r.row_shift = t.row_shift; r.w_cols = t.Q; r.ld_w = t.ld_w; r.dst_w = t.dst_w; r.dst_b = t.dst_b;
            red.r[n_red++] = r;
            max_total = std::max(max_total, t.P * (t.Q + t.n_extra));
        }
        hipError_t err = hipSuccess;
#define MARL_TN(PBW, QBN, PL, ABF, BATCH, COUNT, PPAD, MAXQ) MARL_TN2(PBW, QBN, PL, ABF, false, BATCH, COUNT, PPAD, MAXQ)
#define MARL_TN2(PBW, QBN, PL, ABF, BBF, BATCH, COUNT, PPAD, MAXQ)                                       \
    do {                                                                                                 \
        const size_t lds = (size_t)(PL == 1 ? 2 : 1) * PL * (PPAD + MAXQ) * 80;      /* 80 bytes per staged column and plane */ \
        err = allow_large_lds<tn_gemm_kernel<PBW, QBN, PL, ABF, BBF>>(kLdsLimit);                        \
        if (err != hipSuccess) return err;                                                               \
        hipLaunchKernelGGL((tn_gemm_kernel<PBW, QBN, PL, ABF, BBF>), dim3(chunks, COUNT), dim3(kTnThreads), lds, stream, BATCH); \
        err = hipGetLastError();                                                                         \
        if (err != hipSuccess) return err;                                                               \
    } while (0)
        // the element type of A is the same for every product of a call (bf16 adjoints only with one plane)
        const bool a_bf16 = list[done].a.bf16 != 0;
        bool all_wide = planes == 1 && a_bf16;
        for (int i = done; i < taken && all_wide; ++i) all_wide = tn_wide_fits(list[i], M);
        if (a_in_groups && !all_wide) return hipErrorInvalidValue;
#define MARL_TN_WIDE(PBW, QBN, BBF, BATCH, COUNT)                                                         \
    do {                                                                                                 \
        err = allow_large_lds<tn_gemm_wide_kernel<PBW, QBN, BBF>>(kLdsLimit);                            \
        if (err != hipSuccess) return err;                                                               \
        const size_t lds_wide = tn_wide_lds<PBW, QBN>();                                                 \
        hipLaunchKernelGGL((tn_gemm_wide_kernel<PBW, QBN, BBF>), dim3(chunks, COUNT), dim3(kTnThreads), lds_wide, stream, BATCH); \
        err = hipGetLastError();                                                                         \
        if (err != hipSuccess) return err;                                                               \
    } while (0)
        if (all_wide) {
            if (n_wide) {
                if (list[done].b.bf16) MARL_TN_WIDE(3, 9, true, wide, n_wide);
                else MARL_TN_WIDE(3, 9, false, wide, n_wide);
            }
            if (n_narrow) MARL_TN_WIDE(1, 21, false, narrow, n_narrow);
            n_wide = n_narrow = 0;
        }
#undef MARL_TN_WIDE
        if (n_wide) {
            if (planes == 2) MARL_TN(3, 9, 2, false, wide, n_wide, 384, max_q_wide);
            else if (a_bf16 && list[done].b.bf16) MARL_TN2(3, 9, 1, true, true, wide, n_wide, 384, max_q_wide);
            else if (a_bf16) MARL_TN(3, 9, 1, true, wide, n_wide, 384, max_q_wide);
            else MARL_TN(3, 9, 1, false, wide, n_wide, 384, max_q_wide);
        }
        if (n_narrow) {
            if (planes == 2) MARL_TN(1, 21, 2, false, narrow, n_narrow, 128, max_q_narrow);
            else if (a_bf16) MARL_TN(1, 21, 1, true, narrow, n_narrow, 128, max_q_narrow);
            else MARL_TN(1, 21, 1, false, narrow, n_narrow, 128, max_q_narrow);
        }
#undef MARL_TN
#undef MARL_TN2
        hipLaunchKernelGGL(tn_reduce_kernel, dim3((max_total + 255) / 256, n_red), dim3(256), 0, stream, red);
        err = hipGetLastError();
        if (err != hipSuccess) return err;
        for (int i = done; i < taken; ++i)
            if (list[i].extra_mode == kExtraAgent) {
                const TnProduct &t = list[i];
                hipLaunchKernelGGL(bias_from_columns_kernel, dim3((t.P + 255) / 256), dim3(256), 0, stream, t.dst_w, t.P, t.ld_w, t.Q,
                                   t.n_extra, t.dst_b);
                err = hipGetLastError();
                if (err != hipSuccess) return err;
            }
        done = taken;
    }
    return hipSuccess;
}


// The products of `list` (every one fits the wide kernel; same M and chunk), without the sum of their chunks:
// product i's partial sums go to partial[i].  One launch per shape and element type of B.
hipError_t launch_tn_gemms_wide(const TnProduct *list, int count, long M, int chunk, float *const *partial, hipStream_t stream)
{
    const int chunks = (int)((M + chunk - 1) / chunk);
    TnGemmBatch batch[3]{};             // wide with bf16 B, wide, narrow
    int n[3] = {0, 0, 0};
    for (int i = 0; i < count; ++i) {
        const TnProduct &t = list[i];
        TnGemmArgs g{};
        g.a = t.a; g.b = t.b; g.M = (int)M; g.P = t.P; g.Q = t.Q; g.extra_mode = t.extra_mode; g.n_extra = t.n_extra;
        g.N = t.N > 0 ? t.N : 1;
        g.qp = (t.Q + t.n_extra + 15) / 16 * 16;
        g.chunk = chunk;
        auto steps = [&](const RowMap &m, unsigned *next, unsigned *wrap) {
            const long nx = (long)m.ld;
            const long w = m.rows_per_group >= M ? nx : m.group_stride - (long)(m.rows_per_group - 1) * m.ld;
            if (nx < 0 || w < 0 || nx >= (1L << 31) || w >= (1L << 31)) return false;
            *next = (unsigned)nx; *wrap = (unsigned)w;
            return true;
        };
        if (!tn_wide_fits(t, M) || !steps(t.a, &g.next_a, &g.wrap_a) || !steps(t.b, &g.next_b, &g.wrap_b)) return hipErrorInvalidValue;
        const bool is_wide = t.P > 128;
        if ((is_wide && (t.P > 384 || g.qp > 144)) || (!is_wide && g.qp > 336) || (t.b.bf16 && !is_wide)) return hipErrorInvalidValue;
        g.partial = partial[i];
        const int kind = is_wide ? (t.b.bf16 ? 0 : 1) : 2;
        if (n[kind] == kTnBatchMax) return hipErrorInvalidValue;
        batch[kind].g[n[kind]++] = g;
    }
    hipError_t err = hipSuccess;
#define MARL_TN_WIDE(PBW, QBN, BBF, KIND)                                                                 \
    if (n[KIND]) {                                                                                       \
        err = allow_large_lds<tn_gemm_wide_kernel<PBW, QBN, BBF>>(kLdsLimit);                            \
        if (err != hipSuccess) return err;                                                               \
        const size_t lds_wide = tn_wide_lds<PBW, QBN>();                                                 \
        hipLaunchKernelGGL((tn_gemm_wide_kernel<PBW, QBN, BBF>), dim3(chunks, n[KIND]), dim3(kTnThreads), lds_wide, stream, batch[KIND]); \
        err = hipGetLastError();                                                                         \
        if (err != hipSuccess) return err;                                                               \
    }
    MARL_TN_WIDE(3, 9, true, 0)
    MARL_TN_WIDE(3, 9, false, 1)
    MARL_TN_WIDE(1, 21, false, 2)
#undef MARL_TN_WIDE
    return hipSuccess;
}

bool qnet_grad_fits(const NetFrags &net)
{
    return unroll_fused_fits(net) && net.D + net.N <= 336;        // the widest product the gradient kernel stages
}

size_t qnet_grad_workspace_bytes(const NetFrags &net, int B, int T) { return make_plan(net, B, T).bytes; }

// grad: packed like the weights (W1, b1, W_ih, W_hh, b_ih, b_hh, W2, b2), device, fully overwritten.
void qnet_grad_activation_slots(const NetFrags &net, int B, int T, void *workspace, float **h_all, void **x_all)
{
    const Plan plan = make_plan(net, B, T);
    *h_all = reinterpret_cast<float *>(static_cast<char *>(workspace) + plan.off_h);
    *x_all = static_cast<char *>(workspace) + plan.off_x;
}

hipError_t launch_qnet_grad(const NetFrags &net, int B, int T, const float *obs, const int32_t *actions,
                            const uint8_t *filled, const float *grad_q, void *workspace, float *grad, hipStream_t stream,
                            bool activations_kept, const SideStream *side, int n_cu)
{
    const Plan plan = make_plan(net, B, T);
    char *ws = static_cast<char *>(workspace);
    float *h_all = reinterpret_cast<float *>(ws + plan.off_h);
    void *x_all = ws + plan.off_x;
    char *da = ws + plan.off_da, *dpre1 = ws + plan.off_dpre1, *dq = ws + plan.off_dq;
    float *partial = reinterpret_cast<float *>(ws + plan.off_partial);
    const int adj_bf16 = net.planes == 1 ? 1 : 0, adj_bytes = adj_bf16 ? 2 : 4;
    const int N = net.N, D = net.D, A = net.A, H = net.H, S = T + 1;

    // forward pass that keeps x and h, unless the caller's unroll has left them in the workspace
    hipError_t err = hipSuccess;
    if (!activations_kept)
        err = launch_unroll_fused(net, net, false, B, T, nullptr, B, obs, nullptr, actions, nullptr, nullptr, filled,
                                  0.0f, nullptr, nullptr, nullptr, nullptr, stream, kTdSave, nullptr, h_all, x_all);
    if (err != hipSuccess) return err;

    BpttArgs a{};
    a.net = net; a.B = B; a.T = T; a.a16 = plan.a16; a.actions = actions; a.filled = filled; a.grad_q = grad_q;
    a.h_all = h_all; a.x_all = x_all; a.da = da; a.dpre1 = dpre1; a.dq = dq;
    a.carry = reinterpret_cast<float *>(ws + plan.off_carry);
    auto reverse = [&](int t_begin, int t_end, hipStream_t on) {
        a.t_begin = t_begin; a.t_end = t_end;
        if (H == 64 && net.planes == 2) return back_dispatch<64, 2, 4>(a, on);
        if (H == 64 && net.planes == 1) return back_dispatch<64, 1, 4>(a, on);
        if (H == 128 && net.planes == 1) return back_dispatch<128, 1, 8>(a, on);
        return hipErrorInvalidValue;
    };

    // offsets of the tensors in the packed vector
    float *gW1 = grad, *gb1 = gW1 + (size_t)H * (D + N), *gWih = gb1 + H, *gWhh = gWih + (size_t)3 * H * H;
    float *gbih = gWhh + (size_t)3 * H * H, *gbhh = gbih + 3 * H, *gW2 = gbhh + 3 * H, *gb2 = gW2 + (size_t)A * H;
    // The four products over the samples (b, t, n) of slots [t0, t1): every operand's rows come in groups of
    // (t1 - t0) N, one per episode.
    struct Four { TnProduct p[4]; };
    auto products_of = [&](int t0, int t1) {
        const int rows = (t1 - t0) * N;
        const size_t first = (size_t)t0 * N;                                 // rows of an episode before the window
        // (all slots: the adjoint arrays' rows follow one another across episodes, one group)
        const bool whole = t0 == 0 && t1 == T;
        const int rows_adj = whole ? (int)std::min<long>((long)B * N * T, 1 << 30) : rows;
        const RowMap da_i{da + first * 4 * H * adj_bytes, whole ? 0 : (long)T * N * 4 * H, rows_adj, 4 * H, adj_bf16};      // columns n, r, z
        RowMap da_h = da_i; da_h.base = da + (first * 4 * H + H) * adj_bytes;                            // columns r, z, n (hidden side)
        const RowMap x_rows{static_cast<const char *>(x_all) + first * H * adj_bytes, (long)S * N * H, rows, H, adj_bf16};      // stored as the adjoints are
        const RowMap h_prev{h_all + first * H, (long)S * N * H, rows, H, 0};
        const RowMap h_new{h_all + (first + N) * H, (long)S * N * H, rows, H, 0};
        const RowMap pre_rows{dpre1 + first * H * adj_bytes, whole ? 0 : (long)T * N * H, rows_adj, H, adj_bf16};
        const RowMap obs_rows{obs + first * D, (long)S * N * D, rows, D, 0};
        const RowMap dq_rows{dq + first * plan.a16 * adj_bytes, whole ? 0 : (long)T * N * plan.a16, rows_adj, plan.a16, adj_bf16};
        // W_ih and b_ih: the adjoint columns are n, r, z -> parameter rows r, z, n: shift by 2H
        return Four{{
            {da_i, x_rows, 3 * H, H, kExtraOnes, 1, N, 2 * H, H, gWih, gbih},
            {da_h, h_prev, 3 * H, H, kExtraOnes, 1, N, 0, H, gWhh, gbhh},
            {pre_rows, obs_rows, H, D, kExtraAgent, N, N, 0, D + N, gW1, gb1},
            {dq_rows, h_new, A, H, kExtraOnes, 1, N, 0, H, gW2, gb2},
        }};
    };

    // The reverse recurrence is one workgroup per 16 rows: a batch with fewer tiles than compute units leaves the
    // rest of the chip idle for as long as the episodes are.  Then the slots are walked in two launches, and the
    // products over the later half run on a second stream beside the earlier half's recurrence.
    const int tiles = (B * N + 15) / 16, t_mid = T / 2;
    bool split = side && side->stream && net.planes == 1 && T >= 16 && 2 * tiles <= 3 * n_cu / 2;
    Four late{}, early{};
    long m_late = 0, m_early = 0;
    if (split) {
        late = products_of(t_mid, T); early = products_of(0, t_mid);
        m_late = (long)B * N * (T - t_mid); m_early = (long)B * N * t_mid;
        for (int i = 0; i < 4 && split; ++i) split = tn_wide_fits(late.p[i], m_late) && tn_wide_fits(early.p[i], m_early);
    }
    if (!split) {
        err = reverse(0, T, stream);
        if (err != hipSuccess) return err;
        const Four all = products_of(0, T);
        return launch_tn_products(net.planes, all.p, 4, (long)B * N * T, plan.chunk, partial, plan.partial_bytes, stream);
    }
    // the later half's products share the chip with the recurrence, whose workgroups hold half the compute units
    // or less: half as many chunks (every chunk's partial sums are written once and read once more)
    auto chunk_of = [](long m, long most) { const long chunks = std::max<long>(1, std::min<long>(most, (m + 31) / 32)); return (int)(((m + chunks - 1) / chunks + 63) / 64 * 64); };
    // (the earlier half's too: its two GRU products then run side by side, one on each stream, 128 workgroups each;
    // 256 chunks for the first layer's product, which runs last and alone, changed nothing)
    const int chunk_late = chunk_of(m_late, 128), chunk_early = chunk_of(m_early, 128);
    const int chunks_late = (int)((m_late + chunk_late - 1) / chunk_late), chunks_early = (int)((m_early + chunk_early - 1) / chunk_early);
    // a product's partial sums: the later half's chunks, then the earlier half's, summed in that order
    float *part_late[4], *part_early[4];
    TnReduceBatch red{};
    int max_total = 0;
    {
        size_t used = 0;
        for (int i = 0; i < 4; ++i) {
            const TnProduct &t = late.p[i];
            const size_t p_pad = t.P > 128 ? 384 : 128, qp = (size_t)(t.Q + t.n_extra + 15) / 16 * 16;
            part_late[i] = reinterpret_cast<float *>(reinterpret_cast<char *>(partial) + used);
            part_early[i] = part_late[i] + (size_t)chunks_late * p_pad * qp;
            used += (size_t)(chunks_late + chunks_early) * p_pad * qp * sizeof(float);
            TnReduceArgs r{};
            r.partial = part_late[i]; r.chunks = chunks_late + chunks_early; r.P = t.P; r.p_pad = (int)p_pad; r.qp = (int)qp;
            r.Q = t.Q; r.n_extra = t.n_extra; r.extra_mode = t.extra_mode;
            r.row_shift = t.row_shift; r.w_cols = t.Q; r.ld_w = t.ld_w; r.dst_w = t.dst_w; r.dst_b = t.dst_b;
            red.r[i] = r;
            max_total = std::max(max_total, t.P * (t.Q + t.n_extra));
        }
        if (used > plan.partial_bytes) return hipErrorInvalidValue;
    }
    err = reverse(t_mid, T, stream);
    if (err == hipSuccess) err = hipEventRecord(side->fork, stream);
    if (err == hipSuccess) err = hipStreamWaitEvent(side->stream, side->fork, 0);
    if (err == hipSuccess) err = launch_tn_gemms_wide(late.p, 4, m_late, chunk_late, part_late, side->stream);
    if (err == hipSuccess) err = reverse(0, t_mid, stream);
    // the earlier half: W_hh's product follows on the second stream (a second fork: it needs the recurrence's end),
    // the other three on the caller's
    if (err == hipSuccess) err = hipEventRecord(side->fork, stream);
    if (err == hipSuccess) err = hipStreamWaitEvent(side->stream, side->fork, 0);
    if (err == hipSuccess) err = launch_tn_gemms_wide(early.p + 1, 1, m_early, chunk_early, part_early + 1, side->stream);
    if (err == hipSuccess) err = hipEventRecord(side->join, side->stream);
    if (err == hipSuccess) err = launch_tn_gemms_wide(early.p, 1, m_early, chunk_early, part_early, stream);
    if (err == hipSuccess) err = launch_tn_gemms_wide(early.p + 2, 2, m_early, chunk_early, part_early + 2, stream);
    if (err == hipSuccess) err = hipStreamWaitEvent(stream, side->join, 0);
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(tn_reduce_kernel, dim3((max_total + 255) / 256, 4), dim3(256), 0, stream, red);
    err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(bias_from_columns_kernel, dim3((H + 255) / 256), dim3(256), 0, stream, gW1, H, D + N, D, N, gb1);
    return hipGetLastError();
}

}  // namespace marl
