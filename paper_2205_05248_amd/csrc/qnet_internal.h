// Internal definitions shared by the host code and the gfx950 kernels of the
// recurrent Q-network library: the handle, and the device-side view of one
// network whose matrices are stored as MFMA operand fragments.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include <functional>
#include <vector>

#include "../../include/marl_qnet.h"

namespace marl {

// 8 bf16 values = the per-lane share of one 32x16 MFMA operand.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

// Fragment storage.  A matrix W[M][K] (M padded to 32, K padded to 16) is cut
// into fragments of 32 rows x 16 k.  Fragment (mb, kc) holds, for lane l
// (g = l / 32, m = l % 32) and idx = 0..7, W[32 mb + m][perm(16 kc + 8 g + idx)].
// A fragment is P planes (P = 1: the bf16 value; P = 2: bf16 high part, then the
// bf16 of the remainder) of 64 lanes x 8 bf16 = 1 KiB each, planes adjacent.
//
// perm is the identity for the first layer (its input is the observation) and
//   permC(16 kc + 8 g + idx) = 16 kc + 8 (idx / 4) + 4 g + idx % 4
// for layers fed by an MFMA result: that is where the 32x32 accumulator layout
// leaves feature values, so a result converts to the next operand in registers.
struct NetFrags {
    const bf16x8 *act_stream;   // decision step: fc1, GRU (6 matrices), fc2 in order of use (stream_layout.h)
    const bf16x8 *proj_stream;  // input projection: fc1, GRU input matrices in order of use
    const bf16x8 *whh;    // [3][H/32][H/16][P][64]   gates r, z, n
    const bf16x8 *w2;     // [mb2][H/16][P][64]
    // fused unroll: fragments of 16 rows x 32 k for the 16x16x32 MFMA (layout in pack_weights.hip)
    const bf16x8 *w1_16;    // [H/16][ceil(D/32)][P][64]
    const bf16x8 *wih_16;   // [3][H/16][H/32][P][64]
    const bf16x8 *whh_16;   // [3][H/16][H/32][P][64]
    const bf16x8 *w2_16;    // [ceil(A/16)][H/32][P][64]
    // streaming decision step: W1 with the agent-id columns as part of the product, [H/16][ceil((D+N)/32)][P][64]
    const bf16x8 *w1x_16;
    // backward pass: the transposed GRU matrices (H output rows, contraction over the 3H stacked gate
    // units r, z, n) as 16x16x32 fragments [H/16][3H/32][P][64], and fc2 as plain fp32 [A][H]
    const bf16x8 *wihT_16;
    const bf16x8 *whhT_16;
    const float *w2_plain;
    const float *bias1;   // [N][H]   b1 + W1[:, D + n]
    const float *b1_plain; // [H]     b1
    const float *bias_r;  // [H]      b_ir + b_hr
    const float *bias_z;  // [H]      b_iz + b_hz
    const float *bias_in; // [H]
    const float *bias_hn; // [H]
    const float *b2;      // [32 mb2] zero padded
    int N, D, A, H;
    int kc1;              // ceil(D / 16)
    int nc1;              // fc1 chunks in the streams
    int act_chunks, proj_chunks;
    int mb2;              // ceil(A / 32)
    int planes;           // P
};

// Host: build the device image of a network from packed fp32 weights.
// Returns bytes; fills `image` (host) and offsets into `net` relative to base 0.
struct PackedImage {
    void *host;        // malloc'ed image, caller frees
    size_t bytes;
    size_t off_act, off_proj, off_whh, off_w2, off_w1_16, off_wih_16, off_whh_16, off_w2_16, off_w1x_16, off_wihT_16, off_whhT_16, off_w2_plain, off_bias1, off_b1_plain, off_bias_r, off_bias_z, off_bias_in, off_bias_hn, off_b2;
    int kc1, mb2, planes, nc1, act_chunks, proj_chunks;
};

// A second stream of a handle's, with the two events that fork work onto it and join it again.
struct SideStream { hipStream_t stream; hipEvent_t fork, join; };

}  // namespace marl

struct marl_qnet {
    marl_qnet_desc desc;
    size_t n_params;
    void *dev_weights;        // one allocation holding every fragment array and bias table
    size_t dev_weight_bytes;
    marl::NetFrags net;
    void *staging;            // pinned host copy of the image, for marl_qnet_set_weights (allocated on first use)
    hipEvent_t staging_done;  // recorded after the last upload from `staging`
    void *scratch;            // input-projection buffer of marl_unroll_td, grown on demand
    size_t scratch_bytes;
    void *static_scratch;     // this device's address of the library's static buffer (marl_unroll_td_static)
    marl::SideStream side;    // second stream of the backward pass, made with the handle
    int n_cu;                          // compute units of the device
    int kernels;                       // MARL_KERNELS_AUTO / MARL_KERNELS_TILE32
    bool timing;                       // record events around the kernels of each call
    std::vector<hipEvent_t> ev_pool;   // events created so far (reused after a read)
    size_t ev_used;                    // events handed out since the last read
    std::vector<int> timed_calls;      // per recorded call: 2 = decision step (2 events), 3 = unroll (3 events)
    // device-side refresh of the image (marl_qnet_sgd_step), built on first use
    int32_t *repack_map;               // device: source parameter of every 16-bit element of the fragment part
    size_t repack_elems;
    marl::PackedImage layout;          // offsets of the image's arrays (host pointer unused)
};

namespace marl {

bool pack_network(const marl_qnet_desc &desc, const float *host_weights, PackedImage *out);

// W [M rows, K columns, leading dimension ld] -> 16x16x32 A-operand fragments
// [ceil(M/16)][ceil(K/32)][planes][64 lanes][8] bf16, zero padded; plane 1 holds the bf16 remainder.
// use_perm: k order in which a pair of accumulators is the next operand (see mfma16_tile.h).
void pack_frags16(uint16_t *out, const float *W, int M, int K, int ld, bool use_perm, int planes);

// Kernel timing for benchmarks.  While the calling thread has a timer set, the next single-kernel launch made
// through launch_kernel records the kernel's own start and end in the timer's events (an extended launch), so
// that the interval is the kernel's duration and nothing of what precedes it on the stream.
struct KernelTimer { hipEvent_t start, stop; };
extern thread_local const KernelTimer *g_kernel_timer;

template <typename Kernel, typename... Args>
void launch_kernel(Kernel kernel, dim3 grid, dim3 block, size_t lds_bytes, hipStream_t stream, Args... args)
{
    if (g_kernel_timer) {
        const KernelTimer t = *g_kernel_timer;
        g_kernel_timer = nullptr;
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)lds_bytes, stream, t.start, t.stop, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds_bytes, stream, args...);
    }
}

// Shared by the C-ABI source files: records the text marl_last_device_error() returns and
// yields MARL_ERR_DEVICE.
int report_device_error(hipError_t err, const char *what);

// Launchers (kernels.hip).  All enqueue on `stream` and return the HIP status.
// env_index (device, n_listed entries) null: all E environments; else only the listed ones, whose
// rows of the E-environment arrays are read and written.
hipError_t launch_act_step(const NetFrags &net, int E, const int32_t *env_index, int n_listed, const float *obs,
                           const uint8_t *avail, const float *h_in,
                           const uint8_t *reset, const int32_t *step_t, float epsilon, uint64_t seed, float *h_out,
                           int32_t *action, float *q_out, hipStream_t stream);

size_t unroll_scratch_bytes(const NetFrags &net, int B, int T);

// What an unroll launch does with the value of the next slot.  kTdPlain: the masked maximum of the
// evaluating network (next_max, td_target).  The double-estimator target takes two single-network
// launches: kTdSelect with the online network stores, besides q_taken, the index of its best
// available action of slot t + 1 into next_action[b, t, n] (-1: none available) and leaves
// next_max / td_target alone; kTdValue with the target network reads those indices and writes
// next_max / td_target from its own value of that action, and leaves q_taken / q_all alone.
// kTdSave (fused kernels, one network): no TD output at all; the fc1 output x and the hidden state of
// every slot go to x_save / h_save [B, T+1, N, H] for the backward pass (h fp32; x fp32, or bf16 for a one-plane
// network, whose every use of x rounds it to bf16 anyway): x_save[b, s] = x of slot s,
// h_save[b, 0] = 0 and h_save[b, s + 1] = the state after slot s (s < T).
// kTdKeep: kTdPlain (one or two networks, all TD outputs) whose online network also stores x_save / h_save.
enum TdMode : int { kTdPlain = 0, kTdSelect = 1, kTdValue = 2, kTdSave = 3, kTdKeep = 4 };

hipError_t launch_unroll_td(const NetFrags &online, const NetFrags &target, bool two_nets, void *scratch_online,
                            void *scratch_target, int B, int T, const int32_t *episode_index, int pool_episodes,
                            const float *obs, const uint8_t *avail,
                            const int32_t *actions, const float *reward, const uint8_t *terminated,
                            const uint8_t *filled, float gamma, float *q_taken, float *next_max, float *td_target,
                            float *q_all, hipStream_t stream, hipEvent_t between, TdMode mode = kTdPlain,
                            int32_t *next_action = nullptr);

// Fused decision step (act_fused.hip).  `fits` as below; groups_hint = workgroups to spread the
// tiles over (0: one per compute unit).
bool act_fused_fits(const NetFrags &net);
hipError_t launch_act_fused(const NetFrags &net, int E, const int32_t *env_index, int n_listed, int groups_hint,
                            const float *obs, const uint8_t *avail,
                            const float *h_in, const uint8_t *reset, const int32_t *step_t, float epsilon,
                            uint64_t seed, float *h_out, int32_t *action, float *q_out, hipStream_t stream);
// env_index non-null (the indexed call): also the output arrays must fit 32-bit byte offsets.
bool act_fused_indexed_fits(const NetFrags &net, int E);
// and the batch: E N below 2^26 rows (dense and indexed calls)
bool act_fused_rows_fit(const NetFrags &net, int E);

// Streaming decision step (act_stream.hip): `fits` for this network and batch; n_cu = compute units of the device.
// Every array must be 16-byte aligned.
bool act_stream_fits(const NetFrags &net, int E);
hipError_t launch_act_stream(const NetFrags &net, int E, int n_cu, const float *obs, const uint8_t *avail,
                             const float *h_in, const uint8_t *reset, const int32_t *step_t, float epsilon,
                             uint64_t seed, float *h_out, int32_t *action, float *q_out, hipStream_t stream);

// Fused unroll (unroll_fused.hip): no scratch buffer.  `fits` tells whether the network's shape
// fits the kernel's LDS and register budgets; otherwise the two-kernel path above is used.
bool unroll_fused_fits(const NetFrags &net);
// episode_index (device, B entries) null: the input arrays hold the batch itself; else they hold
// pool_episodes episodes and batch position b reads episode episode_index[b].
hipError_t launch_unroll_fused(const NetFrags &online, const NetFrags &target, bool two_nets, int B, int T,
                               const int32_t *episode_index, int pool_episodes, const float *obs, const uint8_t *avail, const int32_t *actions, const float *reward,
                               const uint8_t *terminated, const uint8_t *filled, float gamma, float *q_taken,
                               float *next_max, float *td_target, float *q_all, hipStream_t stream,
                               TdMode mode = kTdPlain, int32_t *next_action = nullptr, float *h_save = nullptr,
                               void *x_save = nullptr);

// Products over samples, C[p][q] = sum_m A[m][p] B[m][q] with fp32 operands in global memory (bptt.hip).
// Row m of an operand lives at base + (m / rows_per_group) * group_stride + (m % rows_per_group) * ld.
// Elements are fp32, or bf16 (bf16 != 0: the left operand A of a one-plane product only, the same for every product
// of a call); group_stride and ld count elements either way.  A's rows must be one group (rows_per_group >= M), and
// the steps from one row to the next (ld; from a group's last row to the next group's first) must lie in [0, 2^31).
struct RowMap {
    const void *base;
    long group_stride;
    int rows_per_group, ld;
    int bf16;
};
// Columns appended to B on the fly: one column of ones, or N one-hot columns of (m % N).
enum ExtraCols : int { kExtraNone = 0, kExtraOnes = 1, kExtraAgent = 2 };
// The samples are cut into chunks of `chunk` (a multiple of 32), one workgroup each and product.  Shapes served:
// P <= 384 with Q + extra <= 144, or P <= 128 with Q + extra <= 336.  planes: 2 = operands as bf16 pairs (three
// MFMAs per product), 1 = rounded to bf16.  The sum of the chunks goes to dst_w[((p + row_shift) % P) * ld_w + q]
// for q < Q (and the agent columns, which continue the row), the column of ones to dst_b[(p + row_shift) % P].
struct TnProduct {
    RowMap a, b;
    int P, Q, extra_mode, n_extra, N, row_shift, ld_w;
    float *dst_w, *dst_b;
};
// tn_partial_bytes: what one product needs of `partial`; launch_tn_products runs the list (same M and chunk for
// all), as many at a time as `partial` holds.
size_t tn_partial_bytes(long M, int chunk, int P, int q_total);
hipError_t launch_tn_products(int planes, const TnProduct *list, int count, long M, int chunk, float *partial,
                              size_t partial_bytes, hipStream_t stream);

// Backward pass (bptt.hip): the gradient of sum(grad_q * q_taken) with respect to the packed parameters.
// `fits`: the network runs on the fused unroll kernel and its widest layer fits the gradient product.
bool qnet_grad_fits(const NetFrags &net);
size_t qnet_grad_workspace_bytes(const NetFrags &net, int B, int T);
// activations_kept: the workspace already holds x and h of this batch (an unroll in kTdKeep mode wrote them to the
// places qnet_grad_activation_slots names); otherwise the call runs its own forward pass first.
void qnet_grad_activation_slots(const NetFrags &net, int B, int T, void *workspace, float **h_all, void **x_all);
// side: a second stream of the handle's, with two events, on which part of the products may run beside the
// recurrence (null: everything on `stream`); n_cu: compute units of the device.
hipError_t launch_qnet_grad(const NetFrags &net, int B, int T, const float *obs, const int32_t *actions,
                            const uint8_t *filled, const float *grad_q, void *workspace, float *grad, hipStream_t stream,
                            bool activations_kept, const SideStream *side, int n_cu);

// Device-side parameter update (repack.hip).  build_repack_map (host): for every 16-bit element of the image's
// fragment part, the parameter it holds; launch_sgd_step: weights -= lr * grad, then the image rebuilt from them.
// probe_fragment_map: the same for any image whose packer is handed in (pack(w, out): the frag_elems 16-bit
// elements of the fragment part packed from w); launch_sgd_and_fragments / launch_copy_refresh: the kernels.
// How the weights move: plain gradient descent (sq_avg null) or RMSprop with the running mean of squares sq_avg.
struct UpdateRule {
    float *sq_avg = nullptr;
    float alpha = 0.0f, eps = 0.0f;
};
using FragPacker = std::function<bool(const float *, uint16_t *)>;
bool probe_fragment_map(size_t n_params, size_t frag_elems, const FragPacker &pack, std::vector<int32_t> *map);
hipError_t launch_sgd_and_fragments(float *weights, const float *grad, float lr, size_t n_params, const int32_t *map_dev,
                                    size_t map_elems, void *image_dev, hipStream_t stream, const UpdateRule &rule = UpdateRule());
hipError_t launch_copy_refresh(const float *weights, const int32_t *src_dev, size_t n, float *dst, hipStream_t stream);
bool build_repack_map(const marl_qnet_desc &desc, size_t n_params, std::vector<int32_t> *map, PackedImage *layout);
bool repack_map_reproduces_packer(const marl_qnet_desc &desc, const float *weights, size_t n_params);
hipError_t launch_sgd_step(const marl_qnet_desc &desc, const PackedImage &layout, int planes, const int32_t *map_dev,
                           size_t map_elems, void *image_dev, float *weights, const float *grad, size_t n_params, float lr,
                           hipStream_t stream, const UpdateRule &rule = UpdateRule());

}  // namespace marl
