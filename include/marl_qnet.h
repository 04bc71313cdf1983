/*
 * marl_qnet.h - C ABI of the batched per-agent recurrent Q-network for MI355X (gfx950).
 *
 * The library evaluates one shared network
 *     x  = ReLU(W1 [obs, onehot(agent)] + b1)
 *     h' = GRUCell(x, h)            (gates r, z, n; n = tanh(W_in x + b_in + r * (W_hn h + b_hn));
 *                                    h' = (1 - z) * n + z * h)
 *     Q  = W2 h' + b2
 * for every agent of every environment, with a hidden state kept separately per
 * agent and per environment (the paper's multidimensional hidden state, Fig. 3,
 * and the passage around it: agents of different environments must not share
 * history).  Two uses:
 *
 *   marl_act_step  - the worker's decision step (Alg. 2, "make decisions based on
 *                    policy, a ~ pi(a|o)"; step 2 of the actor-worker framework):
 *                    one network step for E environments x N agents, then the
 *                    available-action mask and an epsilon-greedy choice.
 *   marl_unroll_td - the forward half of the learner's TD step (Alg. 3, "calculate
 *                    the gradient": y - Q(s, a; theta)) on a batch of B whole
 *                    trajectories (the actor sends whole tracks, Alg. 1): the
 *                    network unrolled over T+1 observation slots, Q of the taken
 *                    actions, the masked maximum of the next slot, and the 1-step
 *                    target y = r + gamma (1 - terminated) max_a' Q_target(t+1, a').
 *
 * Conventions
 *   - "dev" pointers are device memory of the handle's device; "host" pointers
 *     are ordinary host memory.  The caller owns every buffer it passes and keeps
 *     it alive until the stream has run the call.  The library owns the handle,
 *     its device copy of the weights, and a cached scratch buffer (see
 *     marl_unroll_td).
 *   - All arrays are dense, row-major, last index fastest.
 *   - Calls validate their arguments on the host before anything is enqueued,
 *     enqueue on `hip_stream` (a hipStream_t; NULL = the default stream) and
 *     return without synchronising.  Outputs are valid once the stream has
 *     reached the call.
 *   - Return value: 0 on success, a negative MARL_ERR_* otherwise.  Nothing is
 *     written to outputs when an error is returned.  The library never throws or
 *     aborts.
 *   - One handle must not be used by two host threads at once.
 *
 * Packed weights (host, fp32, row-major), Din = obs_dim + n_agents, H = hidden:
 *   W1[H,Din], b1[H], W_ih[3H,H], W_hh[3H,H], b_ih[3H], b_hh[3H], W2[A,H], b2[A];
 *   the three row blocks of W_ih, W_hh, b_ih, b_hh are the gates r, z, n.
 *   Column obs_dim + n of W1 belongs to the one-hot id of agent n.
 */
#ifndef MARL_QNET_H
#define MARL_QNET_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MARL_OK             0
#define MARL_ERR_NULL      -1   /* a required pointer is NULL */
#define MARL_ERR_BAD_DIM   -2   /* a size is <= 0 or outside the supported range */
#define MARL_ERR_BAD_DTYPE -3   /* weight_dtype is not MARL_DTYPE_F32 / MARL_DTYPE_BF16 */
#define MARL_ERR_MISMATCH  -4   /* n_weights != parameter count, or online/target differ */
#define MARL_ERR_BAD_ARG   -5   /* epsilon or gamma outside [0,1] or not finite */
#define MARL_ERR_DEVICE    -6   /* a HIP runtime call failed; see marl_last_device_error */
#define MARL_ERR_NOMEM     -7   /* host or device allocation failed */

#define MARL_DTYPE_F32   0      /* fp32 weights, fp32 accumulation */
#define MARL_DTYPE_BF16  1      /* matrices rounded to bf16 (nearest even) at create; biases, hidden
                                   state and accumulation stay fp32 */

/* Supported ranges (checked by marl_qnet_create). */
#define MARL_MAX_AGENTS   64
#define MARL_MAX_OBS_DIM  1024
#define MARL_MAX_ACTIONS  64
/* hidden must be 64 or 128 */

typedef struct marl_qnet marl_qnet;          /* opaque, library-owned */

typedef struct {
    int32_t n_agents;      /* N */
    int32_t obs_dim;       /* D, without the agent id */
    int32_t n_actions;     /* A */
    int32_t hidden;        /* H */
    int32_t weight_dtype;  /* MARL_DTYPE_* */
    int32_t device;        /* HIP device ordinal */
} marl_qnet_desc;

/* Number of fp32 values in the packed weight vector for desc, 0 if desc is invalid. */
size_t marl_param_count(const marl_qnet_desc *desc);

/*
 * Create a network on desc->device from packed host weights (copied; the caller
 * may free them on return).  n_weights must equal marl_param_count(desc).
 * The description is validated before the device is touched.
 */
int marl_qnet_create(const marl_qnet_desc *desc, const float *host_weights, size_t n_weights,
                     marl_qnet **out);

/*
 * Replace the weights of a network in place (the learner publishing new parameters to the
 * worker's copy; Sec. "Learner" and Alg. 3, the periodic parameter copy).  host_weights: the same
 * packed fp32 layout and count as at create.  The call converts on the host into a pinned staging
 * buffer the handle owns and enqueues one host-to-device copy on hip_stream, so it is ordered
 * like a kernel on that stream: calls enqueued earlier on the stream use the old weights, calls
 * enqueued later the new ones.  Work on other streams is not ordered against it; that is the
 * caller's business.  A second call waits on the host until the previous call's copy has left
 * the staging buffer.  host_weights may be reused as soon as the call returns.
 */
int marl_qnet_set_weights(marl_qnet *q, const float *host_weights, size_t n_weights, void *hip_stream);

/* Writes to *out (host) a copy of the description the handle was created with.  MARL_ERR_NULL for a null argument. */
int marl_qnet_get_desc(const marl_qnet *q, marl_qnet_desc *out);

/*
 * Decision step for E environments (worker, Alg. 2).
 *   obs     dev [E,N,D] f32      observations
 *   avail   dev [E,N,A] u8       1 = action available, 0 = not
 *   h_in    dev [E,N,H] f32      hidden state before the step
 *   reset   dev [E] u8 or NULL   1 = environment e starts an episode: h_in[e] is read as zero
 *   step_t  dev [E] i32          step counter of environment e (environments run asynchronously,
 *                                so each has its own); only feeds the random-number key
 *   epsilon in [0,1]; seed any 64-bit value
 *   h_out   dev [E,N,H] f32      hidden state after the step; may be the same buffer as h_in
 *   action  dev [E,N] i32        chosen action
 *   q_out   dev [E,N,A] f32 or NULL   unmasked Q values
 *
 * Action rule.  greedy = lowest index among the maxima of Q over available
 * actions.  Random numbers are SplitMix64 outputs: S(v) = mix(v + 0x9E3779B97F4A7C15);
 * key = S(S(S(S(seed) ^ e) ^ n) ^ step_t[e]) (step_t taken as its unsigned 32-bit
 * pattern), r1 = S(key), r2 = S(key + 0x9E3779B97F4A7C15).  Explore iff
 * (float)(r1 >> 40) * 2^-24 < epsilon (fp32 compare); the explored action is the
 * j-th available one in ascending order, j = ((r2 >> 32) * c) >> 32, c = number
 * of available actions.  With no available action the result is action 0.
 */
int marl_act_step(marl_qnet *q, int32_t E,
                  const float *obs, const uint8_t *avail, const float *h_in,
                  const uint8_t *reset, const int32_t *step_t,
                  float epsilon, uint64_t seed,
                  float *h_out, int32_t *action, float *q_out, void *hip_stream);

/*
 * Decision step for a sub-batch: only the environments listed in env_index are served (the
 * paper's actors run asynchronously and a worker decides for whichever environments have
 * delivered a new observation; Sec. "Actor-worker" framework, Alg. 2).
 *   env_index dev [n_listed] i32   environments to serve, each in [0, E), no duplicates, any order
 * Every other array is the same E-environment array marl_act_step takes; only the rows of the
 * listed environments are read and written (h_out may be h_in: the hidden states are then a table
 * updated in place, one row per agent of a served environment).  The random-number key uses the
 * environment's own index e, so a listed environment gets exactly the action marl_act_step over
 * all E environments would give it.  An index outside [0, E) is clamped into the range (the call
 * cannot check device data); duplicates make the duplicated rows' outputs unspecified.
 * n_listed = 0 is a no-op.  Kernel family as marl_act_step chooses it (fused16 where the network
 * fits and E N n_actions 4 < 2^31, else tile32; the streaming kernel serves the dense call only).
 * Errors as marl_act_step, plus MARL_ERR_BAD_DIM for n_listed < 0 or n_listed > E.
 */
int marl_act_step_indexed(marl_qnet *q, int32_t E, const int32_t *env_index, int32_t n_listed,
                          const float *obs, const uint8_t *avail, const float *h_in,
                          const uint8_t *reset, const int32_t *step_t, float epsilon, uint64_t seed,
                          float *h_out, int32_t *action, float *q_out, void *hip_stream);

/*
 * Unroll over a batch of B trajectories of T transitions and form TD targets
 * (learner, Alg. 3).  online and target must have equal descriptions and live on
 * the same device; target may be the same handle as online.
 *   obs        dev [B,T+1,N,D] f32
 *   avail      dev [B,T+1,N,A] u8
 *   actions    dev [B,T,N] i32      taken actions, each in [0,A)
 *   reward     dev [B,T] f32        team reward
 *   terminated dev [B,T] u8         1 = the episode truly ended at this transition (no bootstrap)
 *   filled     dev [B,T] u8         1 = real transition, 0 = padding
 *   gamma in [0,1]
 *   q_taken    dev [B,T,N] f32      filled * Q_online(t)[action]
 *   next_max   dev [B,T,N] f32      filled * max over available a of Q_target(t+1)[a] (0 if none)
 *   td_target  dev [B,T,N] f32      filled * (reward + gamma * (1 - terminated) * that maximum)
 *   q_all      dev [B,T+1,N,A] f32 or NULL   Q_online at every slot, unmasked
 * Both networks start from a zero hidden state at slot 0 and keep stepping
 * through padding.  Actions outside [0,A) are clamped into range.
 *
 * Two implementations exist and compute the same function (see
 * marl_qnet_set_kernels).  The tile32 one writes the input half of the GRU
 * gates for every slot to a scratch buffer and then runs the recurrence; the
 * fused16 one keeps every intermediate on chip and needs no scratch.
 *
 * Scratch (tile32 kernels only): the library keeps one device buffer per
 * handle for intermediate activations, grown (never shrunk) when a call needs
 * more than any earlier call; growing synchronises the device.
 * marl_qnet_reserve_unroll sizes it ahead of time so that later calls up to
 * that size allocate nothing (it does nothing for handles on the fused path).
 */
int marl_unroll_td(marl_qnet *online, marl_qnet *target, int32_t B, int32_t T,
                   const float *obs, const uint8_t *avail, const int32_t *actions,
                   const float *reward, const uint8_t *terminated, const uint8_t *filled,
                   float gamma,
                   float *q_taken, float *next_max, float *td_target, float *q_all,
                   void *hip_stream);

/*
 * marl_unroll_td for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, outputs and checks as marl_unroll_td.  It always runs the tile32
 * kernels (whatever marl_qnet_set_kernels chose), whose scratch - the input half
 * of the GRU gates of every slot, for both networks - lies in a static device
 * array of MARL_STATIC_SCRATCH_BYTES that is part of the library's image on each
 * GPU and stays there until the process ends.  The call itself allocates
 * nothing and frees nothing, on the device or through any library: it launches
 * the two kernels and returns.  It records no timing (marl_qnet_set_timing does
 * not apply to it).
 *   MARL_ERR_BAD_DIM (and a message naming both sizes in marl_last_device_error,
 *   which this call clears on entry) when the batch needs more than the array
 *   holds: per network
 *   ceil(B N / 32) (T+1) 3 (hidden/32) x 2048 bytes (bf16 weights) or 4096 (fp32),
 *   rounded up to 256; twice that when target != online.
 * Every call on a GPU, from any handle, uses that GPU's one array: calls that may
 * overlap in time (different streams, different threads) race and must be
 * ordered by the caller.  Nothing in the array has to start at zero: the first
 * kernel writes every block the second one reads, so the contents left by an
 * earlier, larger call do not matter.
 */
#define MARL_STATIC_SCRATCH_BYTES (64u << 20)
int marl_unroll_td_static(marl_qnet *online, marl_qnet *target, int32_t B, int32_t T,
                          const float *obs, const uint8_t *avail, const int32_t *actions,
                          const float *reward, const uint8_t *terminated, const uint8_t *filled,
                          float gamma,
                          float *q_taken, float *next_max, float *td_target, float *q_all,
                          void *hip_stream);

/*
 * The same unroll with its inputs read in place from a larger pool of episodes (the learner's
 * experience replay pool, from which Alg. 3 samples B episodes at random): no packed copy of
 * the batch is made.
 *   pool_episodes               episodes the input arrays hold
 *   episode_index dev [B] i32   pool episode of each batch position, each in [0, pool_episodes);
 *                               repeats are allowed (sampling with replacement)
 *   obs, avail, actions, reward, terminated, filled: as above with leading dimension
 *                               pool_episodes instead of B
 *   outputs: as above, leading dimension B (batch position)
 * An index outside the range is clamped into it (the call cannot check device data).
 * MARL_ERR_BAD_DIM when pool_episodes < 1 or pool_episodes (T+1) N max(D, A) >= 2^30.  Otherwise
 * errors, kernel families and scratch as marl_unroll_td (the scratch is sized by B, not by the pool).
 */
int marl_unroll_td_indexed(marl_qnet *online, marl_qnet *target, int32_t pool_episodes,
                           const int32_t *episode_index, int32_t B, int32_t T,
                           const float *obs, const uint8_t *avail, const int32_t *actions,
                           const float *reward, const uint8_t *terminated, const uint8_t *filled,
                           float gamma, float *q_taken, float *next_max, float *td_target,
                           float *q_all, void *hip_stream);

/*
 * The unroll with the double-estimator TD target.  Alg. 3 uses y^total without defining it;
 * marl_unroll_td takes the target network's own maximum, this call lets the online network
 * choose the next action and the target network value it:
 *   a*[b,t,n]  = lowest-index maximiser over available a of Q_online(t+1)[a]   (-1 if none)
 *   next_max   = filled * Q_target(t+1)[a*]                                    (0 if none)
 *   td_target  = filled * (reward + gamma * (1 - terminated) * Q_target(t+1)[a*])
 *   q_taken, q_all: as marl_unroll_td
 *   next_action dev [B,T,N] i32, required: receives a* (written for padding steps too)
 *   episode_index NULL: the input arrays hold the batch itself (pool_episodes is ignored);
 *   else as marl_unroll_td_indexed.
 * The networks run one after the other on the stream (two launches of the single-network
 * kernels, the second reading next_action), in either kernel family; `online` and `target` may
 * be the same handle, and the result then equals marl_unroll_td's.  The choice of a* is made in
 * fp32 on the library's Q values: where two available actions are within rounding of each other
 * another evaluation order may choose the other one.
 * Errors as marl_unroll_td, plus MARL_ERR_NULL for a missing next_action.
 */
int marl_unroll_td_double(marl_qnet *online, marl_qnet *target, int32_t pool_episodes,
                          const int32_t *episode_index, int32_t B, int32_t T,
                          const float *obs, const uint8_t *avail, const int32_t *actions,
                          const float *reward, const uint8_t *terminated, const uint8_t *filled,
                          float gamma, float *q_taken, float *next_max, float *td_target,
                          int32_t *next_action, float *q_all, void *hip_stream);

int marl_qnet_reserve_unroll(marl_qnet *q, int32_t B, int32_t T);

/*
 * The learner's parameter update (Alg. 3: theta <- theta + d theta, here d theta = -lr * gradient) on
 * the device:
 *   weights[p] <- weights[p] - lr * grad_weights[p]      (fp32: the product is rounded, then the difference)
 * and then the network `q` computes with the new weights: its resident image (operand fragments, bias
 * tables) is rebuilt from them by kernels on the stream, with the same rounding as marl_qnet_create, so
 * that `q` afterwards behaves bit for bit like a network created from the new weights.
 *   weights       dev [marl_param_count] f32, in and out: the caller's copy of the parameters, in the
 *                 order of marl_qnet_create (the handle itself keeps no fp32 copy)
 *   grad_weights  dev [marl_param_count] f32, e.g. from marl_qnet_grad
 *   lr            finite; MARL_ERR_BAD_ARG otherwise
 * Stream-ordered like marl_qnet_set_weights: calls enqueued before it see the old weights, calls after
 * it the new ones.  Nothing crosses to the host.  The first call on a handle builds a map of the image
 * on the host and allocates and fills its device copy (synchronous, a few MB); later calls allocate
 * nothing.  To hand the same update to other networks (the actors' copies, a target network), copy
 * `weights` to the host and use marl_qnet_set_weights, or call this on each handle with its own copy.
 */
int marl_qnet_sgd_step(marl_qnet *q, float *weights, const float *grad_weights, float lr,
                       void *hip_stream);

/*
 * The same with RMSprop in place of plain descent:
 *   sq_avg[p]  <- alpha * sq_avg[p] + (1 - alpha) * grad[p]^2
 *   weights[p] <- weights[p] - lr * grad[p] / (sqrt(sq_avg[p]) + eps)
 * every operation rounded to fp32 on its own, in the order written (products before sums), so that a host
 * reference reproduces it bit for bit.  sq_avg: dev [marl_param_count] f32, in and out, the caller's (start it
 * at zero).  alpha in [0,1], eps > 0 and finite, lr finite: MARL_ERR_BAD_ARG otherwise.  Everything else as
 * marl_qnet_sgd_step.
 */
int marl_qnet_rmsprop_step(marl_qnet *q, float *weights, const float *grad_weights, float *sq_avg,
                           float lr, float alpha, float eps, void *hip_stream);

/*
 * Host-only self-check of the map marl_qnet_sgd_step rebuilds the image with: applied to
 * host_weights with the device kernel's arithmetic it must reproduce, bit for bit, the fragment part of
 * the image marl_qnet_create would build.  Touches no GPU.  MARL_OK, MARL_ERR_MISMATCH if it does not
 * (or n_weights is wrong), MARL_ERR_NULL / the descriptor's error otherwise.
 */
int marl_qnet_check_refresh_map(const marl_qnet_desc *desc, const float *host_weights, size_t n_weights);

/*
 * Backward half of the learner step (Alg. 3: "calculate the gradient"): back-propagation through
 * time over the network `q` for a batch of B episodes of T steps.  With q_taken as marl_unroll_td
 * returns it (q_taken[b,t,n] = filled[b,t] * Q(t)[actions[b,t,n]]) and the caller's
 * grad_q_taken[b,t,n] = dL/dq_taken[b,t,n] (for the mixing network: dL/dQ_total times the mixer's
 * derivative with respect to the agent's value),
 *   grad_weights[p] = sum over b,t,n of grad_q_taken[b,t,n] * d q_taken[b,t,n] / d weights[p]
 * for every entry of the packed parameter vector, in the order of marl_qnet_create's weights.
 *   obs           dev [B,T+1,N,D] f32
 *   actions       dev [B,T,N] i32     clamped into [0,A)
 *   filled        dev [B,T] u8        unfilled steps contribute nothing
 *   grad_q_taken  dev [B,T,N] f32
 *   workspace     dev, 256-byte aligned, at least marl_qnet_grad_workspace_bytes(q, B, T) bytes:
 *                 the saved activations, the adjoints and the partial sums; the caller owns it,
 *                 the call allocates nothing, the contents afterwards are unspecified
 *   grad_weights  dev [marl_param_count] f32, overwritten
 * The call enqueues a forward pass that keeps the activations, the time-reversed pass and the
 * weight-gradient products on the stream.  For a bf16 network part of the products may run on a
 * second stream that the handle owns, forked from hip_stream after the later half of the slots
 * and joined to it before the call's last kernels: to the caller everything is ordered as if on
 * hip_stream (work enqueued there afterwards sees the result; a stream capture of hip_stream takes
 * the fork and the join in).  Two calls on one handle must not be enqueued from two host threads at
 * once.  Sums run in a fixed order: the same inputs give the same bits.  Arithmetic: bf16 MFMA products with fp32 accumulation; fp32 networks split every
 * operand into two bf16 parts, bf16 networks round the operands of every product (adjoints, activations) to bf16.
 * Only networks that run on the fused16 kernels are served (see marl_qnet_set_kernels), with
 * D + N <= 336: MARL_ERR_BAD_DIM otherwise, and for B < 1, T < 1, B (T+1) N 4H >= 2^30, or a
 * workspace that is too small; MARL_ERR_BAD_ARG for a misaligned workspace.
 */
int marl_qnet_grad_workspace_bytes(const marl_qnet *q, int32_t B, int32_t T, size_t *bytes);
int marl_qnet_grad(marl_qnet *q, int32_t B, int32_t T,
                   const float *obs, const int32_t *actions, const uint8_t *filled,
                   const float *grad_q_taken, void *workspace, size_t workspace_bytes,
                   float *grad_weights, void *hip_stream);

/*
 * The learner runs the unroll and then the backward pass on the same batch with the same weights; the pair
 * below lets the unroll leave its activations for the backward pass, which then skips its own forward pass.
 *   marl_unroll_td_keep   marl_unroll_td (same arguments, same outputs, bit for bit) whose online network
 *                         also writes x and h of every slot into `workspace` (sized and aligned as for
 *                         marl_qnet_grad with the same B, T); fused16 kernels only (MARL_ERR_BAD_DIM else)
 *   marl_qnet_grad_kept   marl_qnet_grad (same arguments, same result, bit for bit) that trusts `workspace`
 *                         to hold what marl_unroll_td_keep wrote for this q, B, T, obs, with no change of
 *                         q's weights and no other use of the workspace in between (stream order counts)
 */
int marl_unroll_td_keep(marl_qnet *online, marl_qnet *target, int32_t B, int32_t T,
                        const float *obs, const uint8_t *avail, const int32_t *actions,
                        const float *reward, const uint8_t *terminated, const uint8_t *filled,
                        float gamma, float *q_taken, float *next_max, float *td_target, float *q_all,
                        void *workspace, size_t workspace_bytes, void *hip_stream);
int marl_qnet_grad_kept(marl_qnet *q, int32_t B, int32_t T,
                        const float *obs, const int32_t *actions, const uint8_t *filled,
                        const float *grad_q_taken, void *workspace, size_t workspace_bytes,
                        float *grad_weights, void *hip_stream);

/*
 * Choice of the kernel family for calls on this handle (for marl_unroll_td: the `online` handle).
 * Two families compute the same functions:
 *   fused16  tiles of 16 rows, every weight resident on chip, one kernel per call; serves the
 *            networks that fit its on-chip buffers (bf16 weights: obs_dim <= 320; fp32 weights:
 *            hidden = 64 and obs_dim <= 160; for marl_act_step also n_actions >= 4)
 *   tile32   tiles of 32 rows, weights streamed; the unroll is two kernels with a scratch buffer
 *            between them; serves every network
 *   stream16 a second decision-step kernel on tiles of 16 rows (marl_unroll_td runs fused16 with this choice):
 *            every wavefront holds one block of 16 hidden units of all three weight matrices, inputs travel
 *            from global memory into LDS without passing through registers, and tiles are dealt round-robin
 *            over the workgroups.  It serves bf16 weights with obs_dim + n_agents <= 384 and fp32 weights
 *            with hidden = 64 and obs_dim + n_agents <= 192, for batches whose arrays stay below 2^30 bytes
 *            and are 16-byte aligned; a call it cannot serve runs on fused16 / tile32 as under AUTO.  Measured
 *            slower than fused16 on all five workloads, hence not what AUTO picks.
 *   MARL_KERNELS_AUTO     per entry point, fused16 when the network fits it, else tile32 (the default)
 *   MARL_KERNELS_TILE32   always tile32
 *   MARL_KERNELS_FUSED16  always fused16; MARL_ERR_BAD_DIM if the network does not fit it for both
 *                         entry points
 *   MARL_KERNELS_STREAM16 stream16 for marl_act_step, fused16 for the unroll; MARL_ERR_BAD_DIM if the network
 *                         fits neither
 * Returns MARL_ERR_BAD_ARG for any other value.
 */
#define MARL_KERNELS_AUTO 0
#define MARL_KERNELS_TILE32 1
#define MARL_KERNELS_FUSED16 2
#define MARL_KERNELS_STREAM16 3
int marl_qnet_set_kernels(marl_qnet *q, int32_t which);

/* The family an entry point uses for this handle as things stand: MARL_KERNELS_TILE32,
 * MARL_KERNELS_FUSED16 or MARL_KERNELS_STREAM16 (never AUTO).  Negative status for a null handle or an unknown entry. */
#define MARL_ENTRY_ACT_STEP 0
#define MARL_ENTRY_UNROLL_TD 1
int marl_qnet_kernels_in_use(const marl_qnet *q, int32_t entry);

/*
 * Kernel timing for benchmarks.  While timing is enabled on a handle, marl_act_step and
 * marl_unroll_td (the `online` handle's setting counts) time each kernel they launch with HIP
 * events on the caller's stream, for up to MARL_TIMING_MAX_CALLS calls (later calls run untimed).
 * The one-kernel paths (fused16, stream16) launch their kernel with a start and a stop event of its
 * own, so the interval is the kernel's duration alone; the tile32 path records events before,
 * between and after its kernels, which also counts the gaps between them.  marl_qnet_timing_read waits for the recorded events, returns the mean
 * duration in milliseconds of each kernel over the recorded calls, and clears the record:
 *   act_ms      decision-step kernel, over *act_calls calls
 *   unroll_ms   two-kernel path: [0] input-projection kernel, [1] recurrent TD kernel;
 *               fused path: [0] is 0 and [1] the fused kernel; over *unroll_calls calls
 * Means of zero calls are 0.  Event records cost a little stream time; leave timing off in
 * production.  Enabling or disabling clears the record.
 */
#define MARL_TIMING_MAX_CALLS 1024
int marl_qnet_set_timing(marl_qnet *q, int32_t enable);
int marl_qnet_timing_read(marl_qnet *q, float *act_ms, int32_t *act_calls, float unroll_ms[2], int32_t *unroll_calls);

/*
 * Measurement aids for benchmarks: what the current device reaches on two plain kernels, to set next to
 * its nominal peaks.  Not part of the network's path; each call enqueues one kernel and returns.
 *   marl_probe_stream  streams `bytes` (a multiple of 16) from src (dev, 16-byte aligned) with 16-byte loads from
 *                      32 workgroups per compute unit; dst (dev, 16-byte aligned, `bytes` long) non-NULL: copies
 *                      them there (bytes read + bytes written = 2 * bytes); NULL: only reads and sums them.
 *                      sink: dev [1] f32, left alone (it keeps the loads alive).
 *   marl_probe_mfma    two workgroups of four waves per compute unit, each wave issuing iters * 8 independent
 *                      16x16x32 bf16 matrix instructions; *flops (host) receives the floating-point operations the
 *                      launch performs (2 * 16 * 16 * 32 per instruction and wave).
 * MARL_ERR_NULL / MARL_ERR_BAD_DIM (bytes, iters out of range) / MARL_ERR_BAD_ARG (alignment).
 */
int marl_probe_stream(const void *src, void *dst, size_t bytes, float *sink, void *hip_stream);
int marl_probe_mfma(int32_t iters, float *sink, double *flops, void *hip_stream);

/* Free the handle, its weights and scratch.  Synchronises the device.  NULL is allowed. */
int marl_destroy(marl_qnet *q);

/* Static description of a status code. */
const char *marl_strerror(int status);

/* Text of the last HIP error seen by the calling thread ("" if none). */
const char *marl_last_device_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MARL_QNET_H */
