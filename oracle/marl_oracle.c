/*
 * CPU oracle for the batched per-agent recurrent Q-network of the
 * actor-worker-learner framework (worker decision step, Alg. 2; learner TD
 * step, Alg. 3, forward half; per-agent/per-environment hidden state, Fig. 3).
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a slow, plain evaluation of the
 * definitions in double precision with libm, written to be checked against
 * the paper by eye.  It shares no code, header, table or helper with the GPU
 * library, and the GPU library never calls it.
 *
 * Every function works on one (environment, agent) or (episode, agent) pair at
 * a time: the paper requires the hidden state to be kept separately for each
 * agent of each environment at each time step (Sec. "Actor-worker ...
 * Framework", Fig. 3), so the pairs never interact.
 *
 * Pinned by tests that do not call this file to produce their expected values:
 * GRU closed forms on hand-set weights, a library GRUCell, masked-argmax
 * invariants, the published SplitMix64 output sequence, brute-force TD targets.
 * Unpinned by the paper: whole-path values on random weights ("parity
 * unpinned" by any printed number; the paper prints none).
 *
 * Packed weight order (row-major, fp32): W1[H,Din], b1[H], W_ih[3H,H],
 * W_hh[3H,H], b_ih[3H], b_hh[3H], W2[A,H], b2[A]; Din = D + N; gate row blocks
 * of the GRU matrices are r, z, n.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int N, D, A, H, Din;
    const float *W1, *b1, *Wih, *Whh, *bih, *bhh, *W2, *b2;
} net_t;

static void net_bind(net_t *net, int N, int D, int A, int H, const float *w)
{
    net->N = N; net->D = D; net->A = A; net->H = H; net->Din = D + N;
    net->W1 = w;   w += (size_t)H * net->Din;
    net->b1 = w;   w += H;
    net->Wih = w;  w += (size_t)3 * H * H;
    net->Whh = w;  w += (size_t)3 * H * H;
    net->bih = w;  w += 3 * H;
    net->bhh = w;  w += 3 * H;
    net->W2 = w;   w += (size_t)A * H;
    net->b2 = w;
}

long oracle_param_count(int N, int D, int A, int H)
{
    return (long)(D + N) * H + H + 2L * 3 * H * H + 2L * 3 * H + (long)A * H + A;
}

static double sigmoid(double v) { return 1.0 / (1.0 + exp(-v)); }

/*
 * One evaluation of the shared per-agent network for agent n:
 *   x_in = [obs, onehot_N(n)]
 *   x    = max(0, W1 x_in + b1)
 *   r    = sigma(W_ir x + b_ir + W_hr h + b_hr)
 *   z    = sigma(W_iz x + b_iz + W_hz h + b_hz)
 *   nn   = tanh (W_in x + b_in + r * (W_hn h + b_hn))
 *   h'   = (1 - z) * nn + z * h
 *   q    = W2 h' + b2
 * work must hold Din + H + 6H doubles.
 */
static void qnet_eval(const net_t *net, int n, const float *obs, const double *h,
                      double *h_new, double *q, double *work)
{
    const int H = net->H, D = net->D, Din = net->Din, A = net->A;
    double *x_in = work, *x = x_in + Din, *gi = x + H, *gh = gi + 3 * H;

    for (int d = 0; d < D; ++d) x_in[d] = (double)obs[d];
    for (int m = 0; m < net->N; ++m) x_in[D + m] = (m == n) ? 1.0 : 0.0;

    for (int j = 0; j < H; ++j) {
        double s = (double)net->b1[j];
        for (int d = 0; d < Din; ++d) s += (double)net->W1[(size_t)j * Din + d] * x_in[d];
        x[j] = s > 0.0 ? s : 0.0;
    }
    for (int g = 0; g < 3 * H; ++g) {
        double si = (double)net->bih[g], sh = (double)net->bhh[g];
        for (int k = 0; k < H; ++k) {
            si += (double)net->Wih[(size_t)g * H + k] * x[k];
            sh += (double)net->Whh[(size_t)g * H + k] * h[k];
        }
        gi[g] = si; gh[g] = sh;
    }
    for (int j = 0; j < H; ++j) {
        double r = sigmoid(gi[j] + gh[j]);
        double z = sigmoid(gi[H + j] + gh[H + j]);
        double nn = tanh(gi[2 * H + j] + r * gh[2 * H + j]);
        h_new[j] = (1.0 - z) * nn + z * h[j];
    }
    for (int a = 0; a < A; ++a) {
        double s = (double)net->b2[a];
        for (int j = 0; j < H; ++j) s += (double)net->W2[(size_t)a * H + j] * h_new[j];
        q[a] = s;
    }
}

/* Lowest index among the maxima of q over available actions; -1 if none. */
static int masked_argmax(const double *q, const uint8_t *avail, int A)
{
    int best = -1;
    for (int a = 0; a < A; ++a)
        if (avail[a] && (best < 0 || q[a] > q[best])) best = a;
    return best;
}

/* ---- counter-based random numbers: SplitMix64 (Steele, Lea, Flood 2014) ---- */

#define GOLDEN 0x9E3779B97F4A7C15ULL

static uint64_t mix64(uint64_t v)
{
    v ^= v >> 30; v *= 0xBF58476D1CE4E5B9ULL;
    v ^= v >> 27; v *= 0x94D049BB133111EBULL;
    v ^= v >> 31;
    return v;
}

/* One SplitMix64 output: advance the state by the golden gamma, then mix. */
uint64_t oracle_S(uint64_t v) { return mix64(v + GOLDEN); }

/* Two draws for (seed, env, agent, step): key chains the four words through S,
 * then r1, r2 are the first two SplitMix64 outputs of a stream started at key. */
void oracle_rng_draw(uint64_t seed, uint32_t e, uint32_t n, uint32_t t, uint64_t *r1, uint64_t *r2)
{
    uint64_t k = oracle_S(oracle_S(oracle_S(oracle_S(seed) ^ (uint64_t)e) ^ (uint64_t)n) ^ (uint64_t)t);
    *r1 = oracle_S(k);
    *r2 = oracle_S(k + GOLDEN);
}

/* epsilon-greedy over available actions.  u is a 24-bit uniform in [0,1),
 * exact in fp32; the compare with epsilon is an fp32 compare.  The explore
 * pick is integer-only: j = floor(c * (r2 >> 32) / 2^32). */
static int eps_greedy(int greedy, const uint8_t *avail, int A, float epsilon,
                      uint64_t r1, uint64_t r2, uint8_t *explored)
{
    float u = (float)(r1 >> 40) * (1.0f / 16777216.0f);
    int explore = u < epsilon;
    if (explored) *explored = (uint8_t)explore;
    if (!explore) return greedy < 0 ? 0 : greedy;
    uint64_t c = 0;
    for (int a = 0; a < A; ++a) c += avail[a] != 0;
    if (c == 0) return 0;
    uint64_t j = ((r2 >> 32) * c) >> 32;
    for (int a = 0; a < A; ++a)
        if (avail[a] && j-- == 0) return a;
    return 0; /* unreachable: j < c */
}

/* ---- bf16 rounding (round to nearest, ties to even) of an fp32 value ---- */
void oracle_round_bf16(const float *in, float *out, long count)
{
    for (long i = 0; i < count; ++i) {
        uint32_t b; memcpy(&b, &in[i], 4);
        if ((b & 0x7F800000u) == 0x7F800000u) {           /* inf / nan: keep */
            if (b & 0x007FFFFFu) b |= 0x00400000u;
            b &= 0xFFFF0000u;
        } else {
            uint32_t keep = b >> 16, rest = b & 0xFFFFu;
            if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
            b = keep << 16;
        }
        memcpy(&out[i], &b, 4);
    }
}

/* ---- plain thread fan-out over an outer index ---- */
typedef struct { void (*fn)(void *, long); void *ctx; long lo, hi; } span_t;
static void *span_run(void *p)
{
    span_t *s = (span_t *)p;
    for (long i = s->lo; i < s->hi; ++i) s->fn(s->ctx, i);
    return NULL;
}
static void for_each(void (*fn)(void *, long), void *ctx, long count, int nthreads)
{
    if (nthreads < 1) nthreads = 1;
    if (nthreads > count) nthreads = (int)(count > 0 ? count : 1);
    if (nthreads == 1) { span_t s = {fn, ctx, 0, count}; span_run(&s); return; }
    pthread_t *th = malloc(sizeof(pthread_t) * nthreads);
    span_t *sp = malloc(sizeof(span_t) * nthreads);
    for (int i = 0; i < nthreads; ++i) {
        sp[i].fn = fn; sp[i].ctx = ctx;
        sp[i].lo = count * i / nthreads; sp[i].hi = count * (i + 1) / nthreads;
        pthread_create(&th[i], NULL, span_run, &sp[i]);
    }
    for (int i = 0; i < nthreads; ++i) pthread_join(th[i], NULL);
    free(th); free(sp);
}

/* ---------------- act-step (worker decision step, Alg. 2) ---------------- */
typedef struct {
    net_t net; int E;
    const float *obs; const uint8_t *avail; const double *h_in; const uint8_t *reset;
    const int32_t *step_t; float epsilon; uint64_t seed;
    double *h_out; int32_t *action; double *q_out; int32_t *greedy_out; uint8_t *explored;
} act_ctx;

static void act_env(void *p, long e)
{
    act_ctx *c = (act_ctx *)p;
    const net_t *net = &c->net;
    const int N = net->N, D = net->D, A = net->A, H = net->H;
    double *work = malloc(sizeof(double) * (net->Din + 7 * H + H + H + A));
    double *h = work + net->Din + 7 * H, *hn = h + H, *q = hn + H;
    for (int n = 0; n < N; ++n) {
        size_t row = (size_t)e * N + n;
        for (int j = 0; j < H; ++j)
            h[j] = (c->reset && c->reset[e]) ? 0.0 : c->h_in[row * H + j];
        qnet_eval(net, n, c->obs + row * D, h, hn, q, work);
        const uint8_t *av = c->avail + row * A;
        int greedy = masked_argmax(q, av, A);
        uint64_t r1, r2;
        oracle_rng_draw(c->seed, (uint32_t)e, (uint32_t)n, (uint32_t)c->step_t[e], &r1, &r2);
        int act = eps_greedy(greedy, av, A, c->epsilon, r1, r2, c->explored ? &c->explored[row] : NULL);
        memcpy(c->h_out + row * H, hn, sizeof(double) * H);
        memcpy(c->q_out + row * A, q, sizeof(double) * A);
        c->action[row] = act;
        if (c->greedy_out) c->greedy_out[row] = greedy < 0 ? 0 : greedy;
    }
    free(work);
}

/* obs [E,N,D] f32, avail [E,N,A] u8, h_in [E,N,H] f64, reset [E] u8 or NULL,
 * step_t [E] i32 -> h_out [E,N,H] f64, action [E,N] i32, q_out [E,N,A] f64,
 * greedy_out [E,N] i32 or NULL (masked argmax before exploration),
 * explored [E,N] u8 or NULL. */
void oracle_act_step(int N, int D, int A, int H, const float *weights, int E,
                     const float *obs, const uint8_t *avail, const double *h_in,
                     const uint8_t *reset, const int32_t *step_t, float epsilon, uint64_t seed,
                     double *h_out, int32_t *action, double *q_out, int32_t *greedy_out,
                     uint8_t *explored, int nthreads)
{
    act_ctx c;
    net_bind(&c.net, N, D, A, H, weights);
    c.E = E; c.obs = obs; c.avail = avail; c.h_in = h_in; c.reset = reset; c.step_t = step_t;
    c.epsilon = epsilon; c.seed = seed; c.h_out = h_out; c.action = action; c.q_out = q_out;
    c.greedy_out = greedy_out; c.explored = explored;
    for_each(act_env, &c, E, nthreads);
}

/* ------------- unroll + TD (learner step, Alg. 3, forward half) ------------- */
typedef struct {
    net_t online, target; int same; int B, T;
    const float *obs; const uint8_t *avail; const int32_t *actions; const float *reward;
    const uint8_t *terminated, *filled; float gamma;
    double *q_taken, *next_max, *td_target, *q_all;
    const int32_t *row_list; /* optional list of (b*N+n) rows to evaluate */
    int double_q;            /* the next action is chosen by the online network, valued by the target */
    int32_t *next_action;    /* optional [B,T,N]: index of the action whose target value is bootstrapped */
} unroll_ctx;

static void unroll_row(const unroll_ctx *c, int b, int n)
{
    const int N = c->online.N, D = c->online.D, A = c->online.A, H = c->online.H, T = c->T;
    const size_t S = (size_t)T + 1;
    double *work = malloc(sizeof(double) * (c->online.Din + 7 * H));
    double *ho = calloc(2 * H, sizeof(double)), *ht = calloc(2 * H, sizeof(double));
    double *qo = malloc(sizeof(double) * S * A), *qt = qo;
    if (!c->same) qt = malloc(sizeof(double) * S * A);

    /* h_0 = 0 for both networks; Q at every one of the T+1 observation slots */
    for (size_t t = 0; t < S; ++t) {
        const float *o = c->obs + (((size_t)b * S + t) * N + n) * D;
        qnet_eval(&c->online, n, o, ho, ho + H, qo + t * A, work);
        memcpy(ho, ho + H, sizeof(double) * H);
        if (!c->same) {
            qnet_eval(&c->target, n, o, ht, ht + H, qt + t * A, work);
            memcpy(ht, ht + H, sizeof(double) * H);
        }
        if (c->q_all) memcpy(c->q_all + (((size_t)b * S + t) * N + n) * A, qo + t * A, sizeof(double) * A);
    }
    for (int t = 0; t < T; ++t) {
        size_t bt = (size_t)b * T + t, out = bt * N + n;
        double f = c->filled[bt] ? 1.0 : 0.0;
        int u = c->actions[out];
        const uint8_t *av = c->avail + (((size_t)b * S + (t + 1)) * N + n) * A;
        /* plain target: the target network's own best available action at t+1;
         * double estimator: the online network's best available action at t+1 */
        int best = masked_argmax((c->double_q ? qo : qt) + (size_t)(t + 1) * A, av, A);
        if (c->next_action) c->next_action[out] = best;
        double nm = best < 0 ? 0.0 : qt[(size_t)(t + 1) * A + best];
        double y = (double)c->reward[bt] + (double)c->gamma * (c->terminated[bt] ? 0.0 : 1.0) * nm;
        c->q_taken[out] = f * qo[(size_t)t * A + u];
        c->next_max[out] = f * nm;
        c->td_target[out] = f * y;
    }
    if (!c->same) free(qt);
    free(qo); free(ho); free(ht); free(work);
}

static void unroll_episode(void *p, long b)
{
    const unroll_ctx *c = (const unroll_ctx *)p;
    for (int n = 0; n < c->online.N; ++n) unroll_row(c, (int)b, n);
}
static void unroll_listed(void *p, long i)
{
    const unroll_ctx *c = (const unroll_ctx *)p;
    int r = c->row_list[i];
    unroll_row(c, r / c->online.N, r % c->online.N);
}

/* obs [B,T+1,N,D] f32, avail [B,T+1,N,A] u8, actions [B,T,N] i32,
 * reward/terminated/filled [B,T] -> q_taken, next_max, td_target [B,T,N] f64,
 * q_all [B,T+1,N,A] f64 or NULL (online network).  w_target may equal
 * w_online.  If rows != NULL only the n_rows listed (b*N+n) pairs are
 * evaluated and all other output entries are left untouched. */
void oracle_unroll_td(int N, int D, int A, int H, const float *w_online, const float *w_target,
                      int B, int T, const float *obs, const uint8_t *avail, const int32_t *actions,
                      const float *reward, const uint8_t *terminated, const uint8_t *filled,
                      float gamma, double *q_taken, double *next_max, double *td_target,
                      double *q_all, const int32_t *rows, int n_rows, int nthreads)
{
    unroll_ctx c;
    net_bind(&c.online, N, D, A, H, w_online);
    net_bind(&c.target, N, D, A, H, w_target);
    c.same = (w_online == w_target);
    c.B = B; c.T = T; c.obs = obs; c.avail = avail; c.actions = actions; c.reward = reward;
    c.terminated = terminated; c.filled = filled; c.gamma = gamma;
    c.q_taken = q_taken; c.next_max = next_max; c.td_target = td_target; c.q_all = q_all;
    c.row_list = rows;
    c.double_q = 0; c.next_action = NULL;
    if (rows) for_each(unroll_listed, &c, n_rows, nthreads);
    else      for_each(unroll_episode, &c, B, nthreads);
}

/* The double-estimator variant of the TD target.  Alg. 3 writes y^total without
 * defining it; besides the plain reading above (the target network both picks
 * and values the next action) the common alternative is
 *   a* = argmax_{a available at t+1} Q_online(t+1, a)      (lowest index on ties)
 *   next value = Q_target(t+1, a*),   y = r + gamma (1 - terminated) next value
 * Same arrays as oracle_unroll_td; next_max holds the next value and
 * next_action [B,T,N] (optional) the index a*, -1 if no action is available. */
void oracle_unroll_td_double(int N, int D, int A, int H, const float *w_online, const float *w_target,
                             int B, int T, const float *obs, const uint8_t *avail, const int32_t *actions,
                             const float *reward, const uint8_t *terminated, const uint8_t *filled,
                             float gamma, double *q_taken, double *next_max, double *td_target,
                             double *q_all, int32_t *next_action, int nthreads)
{
    unroll_ctx c;
    net_bind(&c.online, N, D, A, H, w_online);
    net_bind(&c.target, N, D, A, H, w_target);
    c.same = (w_online == w_target);
    c.B = B; c.T = T; c.obs = obs; c.avail = avail; c.actions = actions; c.reward = reward;
    c.terminated = terminated; c.filled = filled; c.gamma = gamma;
    c.q_taken = q_taken; c.next_max = next_max; c.td_target = td_target; c.q_all = q_all;
    c.row_list = NULL;
    c.double_q = 1; c.next_action = next_action;
    for_each(unroll_episode, &c, B, nthreads);
}
