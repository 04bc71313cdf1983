/*
 * marl_mixer.h - C ABI of the mixing network of the learner step.
 *
 * The learner (Alg. 3 of arxiv 2205.05248) computes its gradient from
 * (y^total - Q_total(s, a; theta)), where Q_total combines the agents' chosen
 * values under the global state s (state sizes: Table 2).  The per-agent values
 * come from marl_unroll_td (marl_qnet.h); this library evaluates, for a whole
 * batch of episodes in one call,
 *
 *   q_total[b,t] = Mix(theta;  q_taken[b,t,:], state[b,t])
 *   y_total[b,t] = reward[b,t] + gamma (1 - terminated[b,t]) Mix(theta-; next_max[b,t,:], state[b,t+1])
 *   td_err[b,t]  = filled[b,t] ? y_total[b,t] - q_total[b,t] : 0
 *   loss         = ( sum_{b,t} td_err[b,t]^2 ,  number of filled transitions )
 * (the masked mean-squared TD loss the gradient of Alg. 3 descends is loss[0] / loss[1])
 *
 * The paper names the mixer (its experiments train Qmix variants) but prints no
 * equations for it; Mix is the monotonic-mixing definition, in this concrete form
 * (N agents, M hidden units, S state size; |.| keeps the generated weights
 * non-negative, which makes Q_total non-decreasing in every agent's value):
 *
 *   W1[n][m] = | Hw1[n M + m] . s + hb1[n M + m] |
 *   b1[m]    =   Hb1[m] . s + hbb1[m]
 *   w2[m]    = | Hw2[m] . s + hb2[m] |
 *   v        =   sum_m v2[m] relu(V1[m] . s + c1[m]) + c2
 *   Q_total  =   sum_m w2[m] elu( sum_n q[n] W1[n][m] + b1[m] ) + v        elu(x) = x > 0 ? x : exp(x) - 1
 *
 * Packed parameters (host, fp32, row-major, in this order): Hw1[N M, S], hb1[N M],
 * Hb1[M, S], hbb1[M], Hw2[M, S], hb2[M], V1[M, S], c1[M], v2[M], c2[1];
 * marl_mixer_param_count of them.
 *
 * Conventions as in marl_qnet.h: every array argument of marl_mixer_td is a DEVICE
 * pointer to a dense row-major array, owned by the caller, read or written only by
 * work enqueued on `hip_stream` (a hipStream_t, may be null for the default stream);
 * calls validate on the host, enqueue and return without synchronising; the return
 * value is 0 or a negative MARL_ERR_* of marl_qnet.h, and marl_last_device_error()
 * there describes a MARL_ERR_DEVICE.  Nothing is allocated per call.
 */
#ifndef MARL_MIXER_H
#define MARL_MIXER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MARL_MIXER_MAX_STATE_F32  512    /* state_dim limit with fp32 parameters */
#define MARL_MIXER_MAX_STATE_BF16 1024   /* state_dim limit with bf16 parameters */

typedef struct marl_mixer marl_mixer;

typedef struct {
    int32_t n_agents;      /* N, 1 .. 64 */
    int32_t embed;         /* M, hidden units of the mixer: 16, 32 or 64 */
    int32_t state_dim;     /* S, 1 .. the limit above for the dtype */
    int32_t weight_dtype;  /* MARL_DTYPE_F32: fp32 parameters; MARL_DTYPE_BF16: the four state matrices rounded
                              to bf16 (nearest even) at create, everything else fp32; accumulation is fp32 */
    int32_t device;        /* HIP device the handle lives on */
} marl_mixer_desc;

/* (N M + 3 M)(S + 1) + M + 1, or 0 for a descriptor outside the limits. */
size_t marl_mixer_param_count(const marl_mixer_desc *desc);

/* Packs host_weights (n_weights fp32 values in the order above) into the device layout the kernel
 * reads; the host array is not referenced after the call.  MARL_ERR_NULL / _BAD_DIM / _BAD_DTYPE /
 * _MISMATCH (n_weights != parameter count) / _NOMEM / _DEVICE. */
int marl_mixer_create(const marl_mixer_desc *desc, const float *host_weights, size_t n_weights, marl_mixer **out);

/*
 * Replaces the parameters in place (the target mixer taking over the online mixer's parameters, or the
 * learner publishing an update; Alg. 3, last step).  host_weights: the packed layout and count of
 * create.  The call repacks on the host into a pinned staging buffer the handle owns and enqueues one
 * host-to-device copy on hip_stream, so it is ordered like a kernel on that stream: marl_mixer_td calls
 * enqueued earlier use the old parameters, later ones the new.  A second call waits on the host until
 * the previous call's copy has left the staging buffer.  host_weights may be reused on return.
 */
int marl_mixer_set_weights(marl_mixer *m, const float *host_weights, size_t n_weights, void *hip_stream);

/* Frees the handle after the device has finished with it (synchronises).  NULL is a no-op. */
void marl_mixer_destroy(marl_mixer *m);

/*
 * One call over a batch of B episodes of T transitions.
 *   state      [B, T+1, S] f32     global state of every slot
 *   q_taken    [B, T, N]   f32     chosen-action values (online network)
 *   next_max   [B, T, N]   f32     bootstrap values at t+1 (target network)
 *   reward     [B, T]      f32
 *   terminated [B, T]      u8      nonzero: no bootstrap
 *   filled     [B, T]      u8      zero: padding, td_err = 0
 *   q_total, y_total, td_err [B, T] f32 outputs; any of them may be NULL (not written)
 *   loss       [2] f32 output or NULL: sum of squared td_err and number of filled transitions, reduced by
 *              one small second kernel in a fixed order (same bits on every run); needs td_err
 * `target` may equal `online` (or be NULL: the same).  Both handles must have the same
 * descriptor (MARL_ERR_MISMATCH otherwise).  MARL_ERR_BAD_DIM for B < 0, T < 1 or B T >= 2^30;
 * MARL_ERR_BAD_ARG for gamma outside [0, 1]; MARL_ERR_NULL for loss without td_err; B = 0 is a no-op
 * (loss is then left unwritten).
 */
int marl_mixer_td(marl_mixer *online, marl_mixer *target, int32_t B, int32_t T, const float *state,
                  const float *q_taken, const float *next_max, const float *reward, const uint8_t *terminated,
                  const uint8_t *filled, float gamma, float *q_total, float *y_total, float *td_err,
                  float *loss, void *hip_stream);

/*
 * Backward pass of the mixing network (Alg. 3: "calculate the gradient").  With the caller's
 * grad_q_total[b,t] = dL/dQ_total[b,t] (for the masked mean-squared TD loss of marl_mixer_td:
 * -2 td_err / number of filled transitions; y_total is a constant of the target network),
 *   grad_weights[p]     = sum over b,t of grad_q_total[b,t] * d Q_total[b,t] / d weights[p]
 *   grad_q_taken[b,t,n] = grad_q_total[b,t] * d Q_total[b,t] / d q_taken[b,t,n]
 * the second being what marl_qnet_grad takes as its upstream gradient.  d|x|/dx = sign(x) (0 at 0).
 *   state          dev [B,T+1,S] f32   (slot t of each episode is used)
 *   q_taken        dev [B,T,N] f32
 *   grad_q_total   dev [B,T] f32
 *   workspace      dev, 256-byte aligned, at least marl_mixer_grad_workspace_bytes(m, B, T) bytes; the
 *                  caller owns it, the call allocates nothing
 *   grad_q_taken   dev [B,T,N] f32, overwritten
 *   grad_weights   dev [marl_mixer_param_count] f32, overwritten, packed like the weights
 * Sums run in a fixed order.  Arithmetic as the forward pass (bf16 MFMA products, fp32 accumulation; fp32
 * mixers split operands into two bf16 parts).  MARL_ERR_BAD_DIM for B < 1, T < 1, B T ((N + 4) embed + 8) >= 2^30, a
 * workspace that is too small; MARL_ERR_BAD_ARG for a misaligned workspace.
 */
int marl_mixer_grad_workspace_bytes(const marl_mixer *m, int32_t B, int32_t T, size_t *bytes);
int marl_mixer_grad(marl_mixer *m, int32_t B, int32_t T, const float *state, const float *q_taken,
                    const float *grad_q_total, void *workspace, size_t workspace_bytes,
                    float *grad_q_taken, float *grad_weights, void *hip_stream);

/*
 * The learner's parameter update for the mixer on the device, the counterpart of marl_qnet_sgd_step:
 *   weights[p] <- weights[p] - lr * grad_weights[p]      (fp32: the product is rounded, then the difference)
 * and the mixer's resident image is rebuilt from the new weights by kernels on the stream, with the rounding
 * of marl_mixer_create, so that `m` afterwards behaves bit for bit like a mixer created from them.
 *   weights       dev [marl_mixer_param_count] f32, in and out (the caller's copy of the parameters)
 *   grad_weights  dev [marl_mixer_param_count] f32, e.g. from marl_mixer_grad
 *   lr            finite; MARL_ERR_BAD_ARG otherwise
 * Stream-ordered; nothing crosses to the host.  The first call on a handle builds the image's map on the host
 * and allocates and fills its device copy (synchronous); later calls allocate nothing.
 */
int marl_mixer_sgd_step(marl_mixer *m, float *weights, const float *grad_weights, float lr, void *hip_stream);

/* RMSprop in place of plain descent; arguments and arithmetic as marl_qnet_rmsprop_step. */
int marl_mixer_rmsprop_step(marl_mixer *m, float *weights, const float *grad_weights, float *sq_avg,
                            float lr, float alpha, float eps, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif
