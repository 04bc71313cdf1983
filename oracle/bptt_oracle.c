/*
 * CPU oracle for the backward half of the learner step (Alg. 3: "calculate the
 * gradient" of the TD loss with respect to theta): back-propagation through
 * time over the per-agent recurrent Q-network.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  Plain double-precision loops, one
 * (episode, agent) row at a time, written to be checked by eye.  It shares no
 * code, header, table or helper with the GPU library, and the GPU library
 * never calls it.
 *
 * What is computed has a plain definition.  With q_taken[b,t,n] =
 * filled[b,t] * Q_theta(t)[actions[b,t,n]] (the unroll's output) and an
 * upstream array g[b,t,n] = dL/dq_taken[b,t,n] handed in by the caller,
 *     grad[p] = sum_{b,t,n} g[b,t,n] * d q_taken[b,t,n] / d theta[p]
 * for every entry p of the packed parameter vector (order: W1 [H, D+N], b1 [H],
 * W_ih [3H, H], W_hh [3H, H], b_ih [3H], b_hh [3H], W2 [A, H], b2 [A]; gates in
 * the order r, z, n).  The network is the one of the forward oracle:
 *     x  = max(0, W1 [o, onehot(n)] + b1)
 *     r  = sigma(W_ir x + b_ir + W_hr h + b_hr),  z likewise
 *     nn = tanh(W_in x + b_in + r * (W_hn h + b_hn))
 *     h' = (1 - z) nn + z h,   Q = W2 h' + b2,   h = 0 before slot 0.
 * Reverse mode, written out: for t = T-1 .. 0 the adjoint of h'_t is the sum
 * of what flows from Q_t and from step t+1.
 *
 * The ReLU of the first layer makes the gradient of W1 and b1 discontinuous in
 * the forward values: a unit whose pre-activation is within an implementation's
 * forward error of zero may be switched on in one implementation and off in the
 * other, and each is then the exact derivative of what that implementation
 * computed.  For comparing against such an implementation the oracle can also
 * return, per entry of W1 and b1, the ambiguity budget
 *     amb[p] = sum over samples whose pre-activation of that unit lies in
 *              [-delta, delta] of |contribution of the sample to grad[p]|
 * (zero for every other tensor: the switch does not reach them).
 *
 * Pinned by tests that do not call this file for their expected values: a
 * tensor library's automatic differentiation of an independently written
 * forward pass, central finite differences of the forward oracle, closed forms
 * (the output bias, a one-step network by hand), linearity in g.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int N, D, A, H, Din;
    long oW1, ob1, oWih, oWhh, obih, obhh, oW2, ob2, count;
} layout_t;

static void layout(layout_t *L, int N, int D, int A, int H)
{
    L->N = N; L->D = D; L->A = A; L->H = H; L->Din = D + N;
    long o = 0;
    L->oW1 = o;  o += (long)H * L->Din;
    L->ob1 = o;  o += H;
    L->oWih = o; o += 3L * H * H;
    L->oWhh = o; o += 3L * H * H;
    L->obih = o; o += 3 * H;
    L->obhh = o; o += 3 * H;
    L->oW2 = o;  o += (long)A * H;
    L->ob2 = o;  o += A;
    L->count = o;
}

static double sigmoid(double v) { return 1.0 / (1.0 + exp(-v)); }

typedef struct {
    layout_t L; const float *w; int B, T;
    const float *obs; const int32_t *actions; const uint8_t *filled; const double *g;
    double delta;            /* half-width of the band of first-layer pre-activations counted as ambiguous */
} job_t;

/* One (episode, agent) row: forward over slots 0..T-1 keeping every intermediate, then backward. */
static void row_grad(const job_t *J, int b, int n, double *grad, double *amb)
{
    const layout_t *L = &J->L;
    const int H = L->H, D = L->D, Din = L->Din, T = J->T, N = L->N;
    const float *w = J->w;
    const float *W1 = w + L->oW1, *b1 = w + L->ob1, *Wih = w + L->oWih, *Whh = w + L->oWhh;
    const float *bih = w + L->obih, *bhh = w + L->obhh, *W2 = w + L->oW2;
    const size_t S = (size_t)T + 1;
    /* per step: x_in [Din], x [H], h_prev [H], r, z, nn, ghn [H each], h_new [H], pre [H] */
    const size_t per = (size_t)Din + 8 * H;
    double *tape = malloc(sizeof(double) * per * T);
    double *h = calloc(H, sizeof(double));
    for (int t = 0; t < T; ++t) {
        double *x_in = tape + per * t, *x = x_in + Din, *hp = x + H, *r = hp + H, *z = r + H, *nn = z + H,
               *ghn = nn + H, *hn = ghn + H, *pre = hn + H;
        const float *o = J->obs + (((size_t)b * S + t) * N + n) * D;
        for (int d = 0; d < D; ++d) x_in[d] = (double)o[d];
        for (int m = 0; m < N; ++m) x_in[D + m] = (m == n) ? 1.0 : 0.0;
        for (int j = 0; j < H; ++j) {
            double s = (double)b1[j];
            for (int d = 0; d < Din; ++d) s += (double)W1[(size_t)j * Din + d] * x_in[d];
            pre[j] = s;
            x[j] = s > 0.0 ? s : 0.0;
        }
        memcpy(hp, h, sizeof(double) * H);
        for (int j = 0; j < H; ++j) {
            double gi[3], gh[3];
            for (int k3 = 0; k3 < 3; ++k3) {
                const size_t row = (size_t)k3 * H + j;
                double si = (double)bih[row], sh = (double)bhh[row];
                for (int k = 0; k < H; ++k) {
                    si += (double)Wih[row * H + k] * x[k];
                    sh += (double)Whh[row * H + k] * hp[k];
                }
                gi[k3] = si; gh[k3] = sh;
            }
            r[j] = sigmoid(gi[0] + gh[0]);
            z[j] = sigmoid(gi[1] + gh[1]);
            ghn[j] = gh[2];
            nn[j] = tanh(gi[2] + r[j] * gh[2]);
            hn[j] = (1.0 - z[j]) * nn[j] + z[j] * hp[j];
        }
        memcpy(h, hn, sizeof(double) * H);
    }

    double *dh = calloc(H, sizeof(double)), *dh_prev = malloc(sizeof(double) * H);
    double *da = malloc(sizeof(double) * 4 * H);      /* adjoints of the pre-activations: r, z, n (input side), n (hidden side) */
    double *dx = malloc(sizeof(double) * H);
    for (int t = T - 1; t >= 0; --t) {
        const double *x_in = tape + per * t, *x = x_in + Din, *hp = x + H, *r = hp + H, *z = r + H, *nn = z + H,
                     *ghn = nn + H, *hn = ghn + H, *pre = hn + H;
        const size_t bt = (size_t)b * T + t;
        const int u = J->actions[bt * N + n];
        const double gq = J->filled[bt] ? J->g[bt * N + n] : 0.0;        /* adjoint of Q_t[u] */
        /* Q = W2 h' + b2 */
        grad[L->ob2 + u] += gq;
        for (int j = 0; j < H; ++j) {
            grad[L->oW2 + (size_t)u * H + j] += gq * hn[j];
            dh[j] += gq * (double)W2[(size_t)u * H + j];
        }
        /* h' = (1 - z) nn + z h */
        for (int j = 0; j < H; ++j) {
            const double dnn = dh[j] * (1.0 - z[j]);
            const double dz = dh[j] * (hp[j] - nn[j]);
            dh_prev[j] = dh[j] * z[j];
            const double dan = dnn * (1.0 - nn[j] * nn[j]);              /* pre-activation of tanh */
            const double dr = dan * ghn[j];
            da[j] = dr * r[j] * (1.0 - r[j]);
            da[H + j] = dz * z[j] * (1.0 - z[j]);
            da[2 * H + j] = dan;
            da[3 * H + j] = dan * r[j];                                   /* adjoint of W_hn h + b_hn */
        }
        memset(dx, 0, sizeof(double) * H);
        for (int k3 = 0; k3 < 3; ++k3)
            for (int j = 0; j < H; ++j) {
                const size_t row = (size_t)k3 * H + j;
                const double ai = da[row], ah = da[(k3 == 2 ? 3 : k3) * (size_t)H + j];
                grad[L->obih + row] += ai;
                grad[L->obhh + row] += ah;
                for (int k = 0; k < H; ++k) {
                    grad[L->oWih + row * H + k] += ai * x[k];
                    grad[L->oWhh + row * H + k] += ah * hp[k];
                    dx[k] += ai * (double)Wih[row * H + k];
                    dh_prev[k] += ah * (double)Whh[row * H + k];
                }
            }
        /* x = max(0, W1 x_in + b1) */
        for (int j = 0; j < H; ++j) {
            const double dp = x[j] > 0.0 ? dx[j] : 0.0;
            grad[L->ob1 + j] += dp;
            for (int d = 0; d < Din; ++d) grad[L->oW1 + (size_t)j * Din + d] += dp * x_in[d];
            if (amb && fabs(pre[j]) <= J->delta) {
                amb[L->ob1 + j] += fabs(dx[j]);
                for (int d = 0; d < Din; ++d) amb[L->oW1 + (size_t)j * Din + d] += fabs(dx[j] * x_in[d]);
            }
        }
        memcpy(dh, dh_prev, sizeof(double) * H);
    }
    free(dx); free(da); free(dh_prev); free(dh); free(h); free(tape);
}

typedef struct { const job_t *J; int lo, hi; double *grad, *amb; } span_t;
static void *span_run(void *p)
{
    span_t *s = (span_t *)p;
    for (int b = s->lo; b < s->hi; ++b)
        for (int n = 0; n < s->J->L.N; ++n) row_grad(s->J, b, n, s->grad, s->amb);
    return NULL;
}

long bptt_param_count(int N, int D, int A, int H)
{
    layout_t L;
    layout(&L, N, D, A, H);
    return L.count;
}

/* obs [B,T+1,N,D] f32, actions [B,T,N] i32, filled [B,T] u8, g [B,T,N] f64 -> grad [param count] f64,
 * and, if amb != NULL, the ambiguity budget [param count] f64 for the band |pre-activation| <= delta.
 * Episodes are split over threads; each thread sums its rows in order, the threads' sums are
 * added in thread order. */
void bptt_qnet_grad(int N, int D, int A, int H, const float *weights, int B, int T, const float *obs,
                    const int32_t *actions, const uint8_t *filled, const double *g, double *grad,
                    double delta, double *amb, int nthreads)
{
    job_t J;
    layout(&J.L, N, D, A, H);
    J.w = weights; J.B = B; J.T = T; J.obs = obs; J.actions = actions; J.filled = filled; J.g = g;
    J.delta = delta;
    if (nthreads < 1) nthreads = 1;
    if (nthreads > B) nthreads = B > 0 ? B : 1;
    span_t *spans = malloc(sizeof(span_t) * nthreads);
    pthread_t *th = malloc(sizeof(pthread_t) * nthreads);
    for (int i = 0; i < nthreads; ++i) {
        spans[i].J = &J;
        spans[i].lo = (int)((long)B * i / nthreads);
        spans[i].hi = (int)((long)B * (i + 1) / nthreads);
        spans[i].grad = calloc(J.L.count, sizeof(double));
        spans[i].amb = amb ? calloc(J.L.count, sizeof(double)) : NULL;
        pthread_create(&th[i], NULL, span_run, &spans[i]);
    }
    memset(grad, 0, sizeof(double) * J.L.count);
    if (amb) memset(amb, 0, sizeof(double) * J.L.count);
    for (int i = 0; i < nthreads; ++i) {
        pthread_join(th[i], NULL);
        for (long p = 0; p < J.L.count; ++p) grad[p] += spans[i].grad[p];
        if (amb) for (long p = 0; p < J.L.count; ++p) amb[p] += spans[i].amb[p];
        free(spans[i].grad); free(spans[i].amb);
    }
    free(th); free(spans);
}
