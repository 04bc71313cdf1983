/*
 * CPU oracle for the monotonic mixing network that turns the per-agent values
 * of the learner's batch into Q_total and the target y^total of Alg. 3
 * (learner: "calculate the gradient" uses (y^total - Q_total)).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  Plain double-precision evaluation with
 * libm, one transition at a time, written to be checked by eye.  It shares no
 * code, header, table or helper with the GPU library, and the GPU library
 * never calls it.
 *
 * The paper names the mixer (its experiments train "Qmix" variants, Sec.
 * Experimental Display) and gives the state sizes (Table 2) but prints no
 * equations for it.  What is evaluated here is the monotonic-mixing
 * definition: Q_total is a two-layer network over the agents' chosen values
 * whose weights are produced from the global state and forced non-negative, so
 * that Q_total never decreases when an agent's value increases.  The concrete
 * form (one linear map per generated weight, absolute value for
 * non-negativity, ELU hidden units, a two-layer state-value offset) is this
 * repository's reading, stated in full below:
 *
 *   W1[n][m] = | Hw1[n M + m] . s + hb1[n M + m] |        n < N, m < M
 *   b1[m]    =   Hb1[m] . s + hbb1[m]
 *   w2[m]    = | Hw2[m] . s + hb2[m] |
 *   v        =   sum_m v2[m] relu(V1[m] . s + c1[m]) + c2
 *   hid[m]   =   elu( sum_n q[n] W1[n][m] + b1[m] )       elu(x) = x > 0 ? x : exp(x) - 1
 *   Q_total  =   sum_m w2[m] hid[m] + v
 *
 * Packed parameter order (row-major, fp32): Hw1[N M, S], hb1[N M], Hb1[M, S],
 * hbb1[M], Hw2[M, S], hb2[M], V1[M, S], c1[M], v2[M], c2[1].
 *
 * Pinned by tests that do not call this file for their expected values:
 * monotonicity in every agent value, closed forms on hand-set parameters (both
 * ELU branches, the absolute values, the state-value offset), one-hot states
 * against explicit column picks, a tensor-library evaluation, brute-force TD
 * targets on tiny inputs.  "Parity unpinned" by any number printed in the
 * paper: it prints none for the mixer.
 */
#include <math.h>
#include <stdint.h>

typedef struct {
    int N, M, S;
    const float *Hw1, *hb1, *Hb1, *hbb1, *Hw2, *hb2, *V1, *c1, *v2, *c2;
} mixer_t;

long mixer_param_count(int N, int M, int S)
{
    return (long)(N * M + 3 * M) * (S + 1) + M + 1;
}

static void mixer_bind(mixer_t *mx, int N, int M, int S, const float *w)
{
    mx->N = N; mx->M = M; mx->S = S;
    mx->Hw1 = w;  w += (long)N * M * S;
    mx->hb1 = w;  w += (long)N * M;
    mx->Hb1 = w;  w += (long)M * S;
    mx->hbb1 = w; w += M;
    mx->Hw2 = w;  w += (long)M * S;
    mx->hb2 = w;  w += M;
    mx->V1 = w;   w += (long)M * S;
    mx->c1 = w;   w += M;
    mx->v2 = w;   w += M;
    mx->c2 = w;
}

static double dot_state(const float *row, const float *s, int S)
{
    double acc = 0.0;
    for (int k = 0; k < S; ++k) acc += (double)row[k] * (double)s[k];
    return acc;
}

/* Q_total of one transition: q[N] the agents' values, s[S] the global state. */
static double mix(const mixer_t *mx, const double *q, const float *s)
{
    const int N = mx->N, M = mx->M, S = mx->S;
    double total = 0.0;
    for (int m = 0; m < M; ++m) {
        double pre = dot_state(mx->Hb1 + (long)m * S, s, S) + (double)mx->hbb1[m];
        for (int n = 0; n < N; ++n) {
            const long f = (long)n * M + m;
            pre += q[n] * fabs(dot_state(mx->Hw1 + f * S, s, S) + (double)mx->hb1[f]);
        }
        const double hid = pre > 0.0 ? pre : exp(pre) - 1.0;
        total += fabs(dot_state(mx->Hw2 + (long)m * S, s, S) + (double)mx->hb2[m]) * hid;
    }
    double v = (double)mx->c2[0];
    for (int m = 0; m < M; ++m) {
        const double a = dot_state(mx->V1 + (long)m * S, s, S) + (double)mx->c1[m];
        v += (double)mx->v2[m] * (a > 0.0 ? a : 0.0);
    }
    return total + v;
}

/* One mixer on a list of R (values, state) pairs: q [R, N] doubles, s [R, S]. */
void mixer_forward(int N, int M, int S, const float *w, long R, const double *q, const float *s, double *q_total)
{
    mixer_t mx;
    mixer_bind(&mx, N, M, S, w);
    for (long r = 0; r < R; ++r) q_total[r] = mix(&mx, q + r * N, s + r * S);
}

/*
 * The learner's use (Alg. 3): for every transition (b, t)
 *   q_total = Mix(theta;  q_taken[b, t, :], state[b, t])
 *   y_total = reward + gamma (1 - terminated) Mix(theta-; next_max[b, t, :], state[b, t + 1])
 *   td_err  = filled ? y_total - q_total : 0
 * and over the batch  loss[0] = sum td_err^2,  loss[1] = number of filled transitions
 * (the masked mean-squared TD loss is loss[0] / loss[1]).
 * state [B, T+1, S]; q_taken, next_max [B, T, N] doubles; outputs [B, T] doubles, loss [2].
 */
void mixer_td(int N, int M, int S, const float *w_online, const float *w_target, int B, int T,
              const float *state, const double *q_taken, const double *next_max, const float *reward,
              const uint8_t *terminated, const uint8_t *filled, float gamma,
              double *q_total, double *y_total, double *td_err, double *loss)
{
    loss[0] = 0.0;
    loss[1] = 0.0;
    mixer_t on, tg;
    mixer_bind(&on, N, M, S, w_online);
    mixer_bind(&tg, N, M, S, w_target);
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < T; ++t) {
            const long i = (long)b * T + t;
            const float *s_now = state + ((long)b * (T + 1) + t) * S;
            const float *s_next = s_now + S;
            const double qt = mix(&on, q_taken + i * N, s_now);
            const double boot = mix(&tg, next_max + i * N, s_next);
            const double y = (double)reward[i] + (double)gamma * (terminated[i] ? 0.0 : 1.0) * boot;
            q_total[i] = qt;
            y_total[i] = y;
            td_err[i] = filled[i] ? y - qt : 0.0;
            loss[0] += td_err[i] * td_err[i];
            loss[1] += filled[i] ? 1.0 : 0.0;
        }
}

/*
 * Backward pass of the mixing network (Alg. 3: "calculate the gradient"): with an upstream array
 * e[i] = dL/dQ_total[i] handed in by the caller (for the masked mean-squared TD loss: -2 td_err / count),
 *     grad_w[p]    = sum_i e[i] * d Q_total[i] / d w[p]        for every packed parameter p
 *     grad_q[i][n] = e[i] * d Q_total[i] / d q[i][n]           (what flows on into the agents' networks)
 * for the R = B T transitions i = (b, t) with values q [B, T, N] and state[b, t] of state [B, T+1, S].
 * Reverse mode of the definition above, written out per transition; d|x|/dx = sign(x) (0 at 0),
 * elu'(x) = 1 for x > 0, exp(x) otherwise, relu'(x) = [x > 0].
 *
 * sign and the relu step are discontinuous in the forward values: where a generated weight or an offset
 * unit is within an implementation's forward error of zero, two implementations may switch differently and
 * each is the exact derivative of what it computed.  If amb != NULL it receives, per parameter, the summed
 * magnitude by which the gradient can differ through such switches for values in [-delta, delta] (twice the
 * term for a sign, once for a step); it is zero for v2, c2, and grad_q is continuous.
 */
void mixer_grad(int N, int M, int S, const float *w, int B, int T, const float *state, const double *q,
                const double *e, double *grad_q, double *grad_w, double delta, double *amb)
{
    mixer_t mx;
    mixer_bind(&mx, N, M, S, w);
    const long count = mixer_param_count(N, M, S);
    for (long p = 0; p < count; ++p) grad_w[p] = 0.0;
    if (amb) for (long p = 0; p < count; ++p) amb[p] = 0.0;
    const long oHw1 = 0, ohb1 = oHw1 + (long)N * M * S, oHb1 = ohb1 + (long)N * M, ohbb1 = oHb1 + (long)M * S;
    const long oHw2 = ohbb1 + M, ohb2 = oHw2 + (long)M * S, oV1 = ohb2 + M, oc1 = oV1 + (long)M * S;
    /* the same binding on the gradient vector */
    double *gHw1 = grad_w, *ghb1 = gHw1 + (long)N * M * S, *gHb1 = ghb1 + (long)N * M, *ghbb1 = gHb1 + (long)M * S;
    double *gHw2 = ghbb1 + M, *ghb2 = gHw2 + (long)M * S, *gV1 = ghb2 + M, *gc1 = gV1 + (long)M * S;
    double *gv2 = gc1 + M, *gc2 = gv2 + M;
    for (int b = 0; b < B; ++b)
        for (int t = 0; t < T; ++t) {
            const long i = (long)b * T + t;
            const float *s = state + ((long)b * (T + 1) + t) * S;
            const double *qi = q + i * N;
            const double ei = e[i];
            for (int m = 0; m < M; ++m) {
                /* forward for hidden unit m */
                double pre = dot_state(mx.Hb1 + (long)m * S, s, S) + (double)mx.hbb1[m];
                for (int n = 0; n < N; ++n) {
                    const long f = (long)n * M + m;
                    pre += qi[n] * fabs(dot_state(mx.Hw1 + f * S, s, S) + (double)mx.hb1[f]);
                }
                const double hid = pre > 0.0 ? pre : exp(pre) - 1.0;
                const double gen2 = dot_state(mx.Hw2 + (long)m * S, s, S) + (double)mx.hb2[m];
                const double a = dot_state(mx.V1 + (long)m * S, s, S) + (double)mx.c1[m];
                /* backward */
                const double d_gen2 = ei * hid * (gen2 > 0.0 ? 1.0 : gen2 < 0.0 ? -1.0 : 0.0);
                const double d_pre = ei * fabs(gen2) * (pre > 0.0 ? 1.0 : exp(pre));
                const double d_a = ei * (double)mx.v2[m] * (a > 0.0 ? 1.0 : 0.0);
                gv2[m] += ei * (a > 0.0 ? a : 0.0);
                ghb2[m] += d_gen2;
                ghbb1[m] += d_pre;
                gc1[m] += d_a;
                for (int k = 0; k < S; ++k) {
                    gHw2[(long)m * S + k] += d_gen2 * (double)s[k];
                    gHb1[(long)m * S + k] += d_pre * (double)s[k];
                    gV1[(long)m * S + k] += d_a * (double)s[k];
                }
                if (amb && fabs(gen2) <= delta) {
                    amb[ohb2 + m] += 2.0 * fabs(ei * hid);
                    for (int k = 0; k < S; ++k) amb[oHw2 + (long)m * S + k] += 2.0 * fabs(ei * hid * (double)s[k]);
                }
                if (amb && fabs(a) <= delta) {
                    amb[oc1 + m] += fabs(ei * (double)mx.v2[m]);
                    for (int k = 0; k < S; ++k) amb[oV1 + (long)m * S + k] += fabs(ei * (double)mx.v2[m] * (double)s[k]);
                }
                for (int n = 0; n < N; ++n) {
                    const long f = (long)n * M + m;
                    const double gen1 = dot_state(mx.Hw1 + f * S, s, S) + (double)mx.hb1[f];
                    const double d_gen1 = d_pre * qi[n] * (gen1 > 0.0 ? 1.0 : gen1 < 0.0 ? -1.0 : 0.0);
                    ghb1[f] += d_gen1;
                    for (int k = 0; k < S; ++k) gHw1[f * S + k] += d_gen1 * (double)s[k];
                    if (amb && fabs(gen1) <= delta) {
                        amb[ohb1 + f] += 2.0 * fabs(d_pre * qi[n]);
                        for (int k = 0; k < S; ++k) amb[oHw1 + f * S + k] += 2.0 * fabs(d_pre * qi[n] * (double)s[k]);
                    }
                    if (m == 0) grad_q[i * N + n] = 0.0;
                    grad_q[i * N + n] += d_pre * fabs(gen1);
                }
            }
            gc2[0] += ei;
        }
}
