// C-ABI entry points of the recurrent Q-network library (see include/marl_qnet.h)
// and the first-generation gfx950 kernels behind them.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "../../include/marl_qnet.h"
#include "device_math.h"

namespace marl {

// ------------------------------------------------------------------ device-side view of a network
// All matrices are stored transposed ([in][out]) so that the threads of a wave,
// which own consecutive output features, read consecutive addresses.
struct NetDev {
    const float *W1t;   // [Din][H]
    const float *b1;    // [H]
    const float *Wiht;  // [H][3H]
    const float *Whht;  // [H][3H]
    const float *bih;   // [3H]
    const float *bhh;   // [3H]
    const float *W2t;   // [H][A]
    const float *b2;    // [A]
    int N, D, A, H;
};

constexpr int kTileRows = 16;   // (env, agent) rows per workgroup pass
constexpr int kThreads = 256;

struct TileLds {
    float *xin, *x, *h, *hn, *q;
    int *agent;
};

__device__ __forceinline__ TileLds carve_lds(float *base, int D, int H, int A)
{
    TileLds s;
    s.xin = base;
    s.x = s.xin + kTileRows * D;
    s.h = s.x + kTileRows * H;
    s.hn = s.h + kTileRows * H;
    s.q = s.hn + kTileRows * H;
    s.agent = reinterpret_cast<int *>(s.q + kTileRows * A);
    return s;
}

static size_t tile_lds_bytes(int D, int H, int A)
{
    return sizeof(float) * (size_t)kTileRows * (D + 3 * H + A) + sizeof(int) * kTileRows;
}

// One network step for the kTileRows rows staged in LDS: reads s.xin, s.h, s.agent,
// writes s.x, s.hn, s.q.  Ends with a barrier.
template <int H>
__device__ __forceinline__ void tile_forward(const NetDev &net, const TileLds &s)
{
    constexpr int RG = kThreads / H;          // row groups across the workgroup
    constexpr int RPT = kTileRows / RG;       // rows per thread
    const int D = net.D, A = net.A;
    const int j = threadIdx.x % H, rg = threadIdx.x / H;

    {   // fc1 + ReLU; the one-hot agent id selects one column of W1
        float acc[RPT];
#pragma unroll
        for (int i = 0; i < RPT; ++i)
            acc[i] = net.b1[j] + net.W1t[(size_t)(D + s.agent[rg + i * RG]) * H + j];
        for (int k = 0; k < D; ++k) {
            const float w = net.W1t[(size_t)k * H + j];
#pragma unroll
            for (int i = 0; i < RPT; ++i) acc[i] = fmaf(w, s.xin[(rg + i * RG) * D + k], acc[i]);
        }
#pragma unroll
        for (int i = 0; i < RPT; ++i) s.x[(rg + i * RG) * H + j] = fmaxf(acc[i], 0.0f);
    }
    __syncthreads();
    {   // GRU cell, hidden unit j
        float ar[RPT], az[RPT], ain[RPT], ahn[RPT];
        const float br = net.bih[j] + net.bhh[j], bz = net.bih[H + j] + net.bhh[H + j];
        const float bin = net.bih[2 * H + j], bhn = net.bhh[2 * H + j];
#pragma unroll
        for (int i = 0; i < RPT; ++i) { ar[i] = br; az[i] = bz; ain[i] = bin; ahn[i] = bhn; }
        for (int k = 0; k < H; ++k) {
            const float *wi = net.Wiht + (size_t)k * 3 * H + j;
            const float *wh = net.Whht + (size_t)k * 3 * H + j;
            const float wir = wi[0], wiz = wi[H], win = wi[2 * H];
            const float whr = wh[0], whz = wh[H], whn = wh[2 * H];
#pragma unroll
            for (int i = 0; i < RPT; ++i) {
                const float xv = s.x[(rg + i * RG) * H + k], hv = s.h[(rg + i * RG) * H + k];
                ar[i] = fmaf(wir, xv, fmaf(whr, hv, ar[i]));
                az[i] = fmaf(wiz, xv, fmaf(whz, hv, az[i]));
                ain[i] = fmaf(win, xv, ain[i]);
                ahn[i] = fmaf(whn, hv, ahn[i]);
            }
        }
#pragma unroll
        for (int i = 0; i < RPT; ++i) {
            const int row = rg + i * RG;
            const float r = sigmoidf_fast(ar[i]), z = sigmoidf_fast(az[i]);
            const float n = tanhf_fast(ain[i] + r * ahn[i]);
            s.hn[row * H + j] = (1.0f - z) * n + z * s.h[row * H + j];
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < kTileRows * A; idx += kThreads) {   // fc2
        const int row = idx / A, a = idx % A;
        float acc = net.b2[a];
        for (int k = 0; k < H; ++k) acc = fmaf(net.W2t[(size_t)k * A + a], s.hn[row * H + k], acc);
        s.q[idx] = acc;
    }
    __syncthreads();
}

// Lowest-index maximum of q over the available actions; also returns the availability bits.
__device__ __forceinline__ int masked_argmax(const float *q, const uint8_t *avail, int A,
                                             uint64_t &bits, float &best_q)
{
    int best = -1;
    float bq = 0.0f;
    bits = 0;
    for (int a = 0; a < A; ++a) {
        if (avail[a]) {
            bits |= 1ull << a;
            if (best < 0 || q[a] > bq) { best = a; bq = q[a]; }
        }
    }
    best_q = bq;
    return best;
}

template <int H>
__global__ __launch_bounds__(kThreads) void act_step_kernel(
    NetDev net, int rows, const float *__restrict__ obs, const uint8_t *__restrict__ avail,
    const float *h_in, const uint8_t *__restrict__ reset, const int32_t *__restrict__ step_t,
    float epsilon, uint64_t seed, float *h_out, int32_t *__restrict__ action,
    float *__restrict__ q_out)
{
    extern __shared__ float lds[];
    const int D = net.D, A = net.A, N = net.N;
    const TileLds s = carve_lds(lds, D, H, A);
    const int ntiles = (rows + kTileRows - 1) / kTileRows;

    for (int tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int row0 = tile * kTileRows;
        const int valid = min(kTileRows, rows - row0);
        for (int idx = threadIdx.x; idx < kTileRows * D; idx += kThreads)
            s.xin[idx] = idx < valid * D ? obs[(size_t)row0 * D + idx] : 0.0f;
        for (int idx = threadIdx.x; idx < kTileRows * H; idx += kThreads) {
            float v = 0.0f;
            if (idx < valid * H) {
                const int e = (row0 + idx / H) / N;
                if (!(reset && reset[e])) v = h_in[(size_t)row0 * H + idx];
            }
            s.h[idx] = v;
        }
        if (threadIdx.x < kTileRows) s.agent[threadIdx.x] = threadIdx.x < valid ? (row0 + threadIdx.x) % N : 0;
        __syncthreads();

        tile_forward<H>(net, s);

        for (int idx = threadIdx.x; idx < valid * H; idx += kThreads) h_out[(size_t)row0 * H + idx] = s.hn[idx];
        if (q_out)
            for (int idx = threadIdx.x; idx < valid * A; idx += kThreads) q_out[(size_t)row0 * A + idx] = s.q[idx];
        if (threadIdx.x < valid) {
            const int row = row0 + threadIdx.x, e = row / N, n = row % N;
            uint64_t bits; float bq;
            int greedy = masked_argmax(s.q + threadIdx.x * A, avail + (size_t)row * A, A, bits, bq);
            if (greedy < 0) greedy = 0;
            action[row] = eps_greedy_pick(greedy, bits, epsilon, seed, (uint32_t)e, (uint32_t)n,
                                          (uint32_t)step_t[e]);
        }
        __syncthreads();
    }
}

// grid = (row tiles, 1 or 2).  blockIdx.y = 0 evaluates the online network and
// emits q_taken / q_all; blockIdx.y = 1 (only when the target network is a
// different one) evaluates the target network and emits next_max / td_target.
// With a single network one pass emits everything.
template <int H>
__global__ __launch_bounds__(kThreads) void unroll_td_kernel(
    NetDev online, NetDev target, int two_nets, int B, int T,
    const float *__restrict__ obs, const uint8_t *__restrict__ avail,
    const int32_t *__restrict__ actions, const float *__restrict__ reward,
    const uint8_t *__restrict__ terminated, const uint8_t *__restrict__ filled, float gamma,
    float *__restrict__ q_taken, float *__restrict__ next_max, float *__restrict__ td_target,
    float *__restrict__ q_all)
{
    extern __shared__ float lds[];
    const bool is_target = blockIdx.y == 1;
    const NetDev &net = is_target ? target : online;
    const bool emit_online = !is_target, emit_target = is_target || !two_nets;
    const int D = net.D, A = net.A, N = net.N;
    TileLds s = carve_lds(lds, D, H, A);
    const int rows = B * N;
    const int row0 = blockIdx.x * kTileRows;
    const int valid = min(kTileRows, rows - row0);
    const size_t S = (size_t)T + 1;

    for (int idx = threadIdx.x; idx < kTileRows * H; idx += kThreads) s.h[idx] = 0.0f;
    if (threadIdx.x < kTileRows) s.agent[threadIdx.x] = threadIdx.x < valid ? (row0 + threadIdx.x) % N : 0;

    for (int t = 0; t <= T; ++t) {
        for (int idx = threadIdx.x; idx < kTileRows * D; idx += kThreads) {
            const int r = idx / D, d = idx % D;
            float v = 0.0f;
            if (r < valid) {
                const int row = row0 + r, b = row / N, n = row % N;
                v = obs[(((size_t)b * S + t) * N + n) * D + d];
            }
            s.xin[idx] = v;
        }
        __syncthreads();
        tile_forward<H>(net, s);

        if (emit_online && q_all) {
            for (int idx = threadIdx.x; idx < valid * A; idx += kThreads) {
                const int row = row0 + idx / A, b = row / N, n = row % N;
                q_all[(((size_t)b * S + t) * N + n) * A + idx % A] = s.q[idx];
            }
        }
        if (threadIdx.x < valid) {
            const int row = row0 + threadIdx.x, b = row / N, n = row % N;
            const float *q = s.q + threadIdx.x * A;
            if (emit_online && t < T) {
                const size_t bt = (size_t)b * T + t;
                int u = actions[bt * N + n];
                u = min(max(u, 0), A - 1);
                q_taken[bt * N + n] = filled[bt] ? q[u] : 0.0f;
            }
            if (emit_target && t >= 1) {
                const size_t bt = (size_t)b * T + (t - 1);
                uint64_t bits; float bq;
                masked_argmax(q, avail + (((size_t)b * S + t) * N + n) * A, A, bits, bq);
                const float keep = terminated[bt] ? 0.0f : 1.0f;
                const float y = reward[bt] + gamma * keep * bq;
                const bool f = filled[bt] != 0;
                next_max[bt * N + n] = f ? bq : 0.0f;
                td_target[bt * N + n] = f ? y : 0.0f;
            }
        }
        __syncthreads();
        float *tmp = s.h; s.h = s.hn; s.hn = tmp;
    }
}

}  // namespace marl

// ------------------------------------------------------------------ host side
struct marl_qnet {
    marl_qnet_desc desc;
    size_t n_params;
    float *dev_weights;       // one allocation holding every transposed tensor
    marl::NetDev net;
};

namespace {

thread_local char g_last_error[256] = "";

int device_fail(hipError_t err, const char *what)
{
    std::snprintf(g_last_error, sizeof(g_last_error), "%s: %s", what, hipGetErrorString(err));
    return MARL_ERR_DEVICE;
}
#define MARL_HIP(call)                                            \
    do {                                                          \
        hipError_t e_ = (call);                                   \
        if (e_ != hipSuccess) return device_fail(e_, #call);      \
    } while (0)

bool desc_valid(const marl_qnet_desc *d, int *why)
{
    if (d->n_agents < 1 || d->n_agents > MARL_MAX_AGENTS || d->obs_dim < 1 || d->obs_dim > MARL_MAX_OBS_DIM ||
        d->n_actions < 1 || d->n_actions > MARL_MAX_ACTIONS || (d->hidden != 64 && d->hidden != 128) ||
        d->device < 0) {
        *why = MARL_ERR_BAD_DIM;
        return false;
    }
    if (d->weight_dtype != MARL_DTYPE_F32 && d->weight_dtype != MARL_DTYPE_BF16) {
        *why = MARL_ERR_BAD_DTYPE;
        return false;
    }
    return true;
}

size_t param_count(const marl_qnet_desc *d)
{
    const size_t H = d->hidden, Din = (size_t)d->obs_dim + d->n_agents, A = d->n_actions;
    return Din * H + H + 2 * 3 * H * H + 2 * 3 * H + A * H + A;
}

// fp32 -> nearest bf16 (ties to even), returned as the fp32 value it represents.
float round_to_bf16(float v)
{
    uint32_t b;
    std::memcpy(&b, &v, 4);
    if ((b & 0x7F800000u) == 0x7F800000u) {
        if (b & 0x007FFFFFu) b |= 0x00400000u;
        b &= 0xFFFF0000u;
    } else {
        b += 0x7FFFu + ((b >> 16) & 1u);
        b &= 0xFFFF0000u;
    }
    std::memcpy(&v, &b, 4);
    return v;
}

struct DeviceGuard {
    int prev = -1;
    bool ok = false;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) == hipSuccess && hipSetDevice(dev) == hipSuccess) ok = true;
    }
    ~DeviceGuard()
    {
        if (ok && prev >= 0) (void)hipSetDevice(prev);
    }
};

bool unit_interval(float v) { return std::isfinite(v) && v >= 0.0f && v <= 1.0f; }

}  // namespace

extern "C" {

size_t marl_param_count(const marl_qnet_desc *desc)
{
    int why;
    if (!desc || !desc_valid(desc, &why)) return 0;
    return param_count(desc);
}

int marl_qnet_create(const marl_qnet_desc *desc, const float *host_weights, size_t n_weights, marl_qnet **out)
{
    if (!desc || !host_weights || !out) return MARL_ERR_NULL;
    int why;
    if (!desc_valid(desc, &why)) return why;
    if (n_weights != param_count(desc)) return MARL_ERR_MISMATCH;

    const int N = desc->n_agents, D = desc->obs_dim, A = desc->n_actions, H = desc->hidden, Din = D + N;
    const bool bf16 = desc->weight_dtype == MARL_DTYPE_BF16;
    auto mat = [&](float v) { return bf16 ? round_to_bf16(v) : v; };

    // Transpose every matrix into [in][out]; biases are copied as they are.
    std::vector<float> t(n_weights);
    const float *W1 = host_weights, *b1 = W1 + (size_t)H * Din, *Wih = b1 + H, *Whh = Wih + (size_t)3 * H * H;
    const float *bih = Whh + (size_t)3 * H * H, *bhh = bih + 3 * H, *W2 = bhh + 3 * H, *b2 = W2 + (size_t)A * H;
    size_t off = 0;
    const size_t oW1t = off; off += (size_t)Din * H;
    const size_t ob1 = off; off += H;
    const size_t oWiht = off; off += (size_t)3 * H * H;
    const size_t oWhht = off; off += (size_t)3 * H * H;
    const size_t obih = off; off += 3 * H;
    const size_t obhh = off; off += 3 * H;
    const size_t oW2t = off; off += (size_t)A * H;
    const size_t ob2 = off; off += A;
    for (int j = 0; j < H; ++j)
        for (int k = 0; k < Din; ++k) t[oW1t + (size_t)k * H + j] = mat(W1[(size_t)j * Din + k]);
    for (int g = 0; g < 3 * H; ++g)
        for (int k = 0; k < H; ++k) {
            t[oWiht + (size_t)k * 3 * H + g] = mat(Wih[(size_t)g * H + k]);
            t[oWhht + (size_t)k * 3 * H + g] = mat(Whh[(size_t)g * H + k]);
        }
    for (int a = 0; a < A; ++a)
        for (int k = 0; k < H; ++k) t[oW2t + (size_t)k * A + a] = mat(W2[(size_t)a * H + k]);
    std::memcpy(&t[ob1], b1, sizeof(float) * H);
    std::memcpy(&t[obih], bih, sizeof(float) * 3 * H);
    std::memcpy(&t[obhh], bhh, sizeof(float) * 3 * H);
    std::memcpy(&t[ob2], b2, sizeof(float) * A);

    marl_qnet *q = new (std::nothrow) marl_qnet();
    if (!q) return MARL_ERR_NOMEM;
    q->desc = *desc;
    q->n_params = n_weights;
    q->dev_weights = nullptr;

    int n_dev = 0;
    hipError_t err = hipGetDeviceCount(&n_dev);
    if (err != hipSuccess || desc->device >= n_dev) {
        delete q;
        if (err != hipSuccess) return device_fail(err, "hipGetDeviceCount");
        std::snprintf(g_last_error, sizeof(g_last_error), "device %d not present (%d devices)", desc->device, n_dev);
        return MARL_ERR_DEVICE;
    }
    DeviceGuard guard(desc->device);
    if (!guard.ok) { delete q; return device_fail(hipErrorInvalidDevice, "hipSetDevice"); }
    err = hipMalloc(&q->dev_weights, sizeof(float) * n_weights);
    if (err != hipSuccess) { delete q; return err == hipErrorOutOfMemory ? MARL_ERR_NOMEM : device_fail(err, "hipMalloc"); }
    err = hipMemcpy(q->dev_weights, t.data(), sizeof(float) * n_weights, hipMemcpyHostToDevice);
    if (err != hipSuccess) { (void)hipFree(q->dev_weights); delete q; return device_fail(err, "hipMemcpy"); }

    float *w = q->dev_weights;
    q->net = marl::NetDev{w + oW1t, w + ob1, w + oWiht, w + oWhht, w + obih, w + obhh, w + oW2t, w + ob2, N, D, A, H};
    *out = q;
    return MARL_OK;
}

int marl_qnet_get_desc(const marl_qnet *q, marl_qnet_desc *out)
{
    if (!q || !out) return MARL_ERR_NULL;
    *out = q->desc;
    return MARL_OK;
}

int marl_act_step(marl_qnet *q, int32_t E, const float *obs, const uint8_t *avail, const float *h_in,
                  const uint8_t *reset, const int32_t *step_t, float epsilon, uint64_t seed,
                  float *h_out, int32_t *action, float *q_out, void *hip_stream)
{
    if (!q) return MARL_ERR_NULL;
    if (E < 0 || (int64_t)E * q->desc.n_agents > (int64_t)1 << 30) return MARL_ERR_BAD_DIM;
    if (!unit_interval(epsilon)) return MARL_ERR_BAD_ARG;
    if (E == 0) return MARL_OK;
    if (!obs || !avail || !h_in || !step_t || !h_out || !action) return MARL_ERR_NULL;

    DeviceGuard guard(q->desc.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    const marl::NetDev &net = q->net;
    const int rows = E * net.N;
    const int ntiles = (rows + marl::kTileRows - 1) / marl::kTileRows;
    const size_t lds = marl::tile_lds_bytes(net.D, net.H, net.A);
    const dim3 grid((unsigned)ntiles), block(marl::kThreads);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (net.H == 64)
        hipLaunchKernelGGL(marl::act_step_kernel<64>, grid, block, lds, stream, net, rows, obs, avail, h_in, reset,
                           step_t, epsilon, seed, h_out, action, q_out);
    else
        hipLaunchKernelGGL(marl::act_step_kernel<128>, grid, block, lds, stream, net, rows, obs, avail, h_in, reset,
                           step_t, epsilon, seed, h_out, action, q_out);
    MARL_HIP(hipGetLastError());
    return MARL_OK;
}

int marl_qnet_reserve_unroll(marl_qnet *q, int32_t B, int32_t T)
{
    if (!q) return MARL_ERR_NULL;
    if (B < 0 || T < 1) return MARL_ERR_BAD_DIM;
    return MARL_OK;   // the current kernels keep every intermediate on chip
}

int marl_unroll_td(marl_qnet *online, marl_qnet *target, int32_t B, int32_t T, const float *obs,
                   const uint8_t *avail, const int32_t *actions, const float *reward,
                   const uint8_t *terminated, const uint8_t *filled, float gamma, float *q_taken,
                   float *next_max, float *td_target, float *q_all, void *hip_stream)
{
    if (!online || !target) return MARL_ERR_NULL;
    const marl_qnet_desc &a = online->desc, &b = target->desc;
    if (a.n_agents != b.n_agents || a.obs_dim != b.obs_dim || a.n_actions != b.n_actions || a.hidden != b.hidden ||
        a.weight_dtype != b.weight_dtype || a.device != b.device)
        return MARL_ERR_MISMATCH;
    if (B < 0 || T < 1 || (int64_t)B * a.n_agents > (int64_t)1 << 30 || (int64_t)T > (int64_t)1 << 20) return MARL_ERR_BAD_DIM;
    if (!unit_interval(gamma)) return MARL_ERR_BAD_ARG;
    if (B == 0) return MARL_OK;
    if (!obs || !avail || !actions || !reward || !terminated || !filled || !q_taken || !next_max || !td_target)
        return MARL_ERR_NULL;

    DeviceGuard guard(a.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    const marl::NetDev &net = online->net;
    const int rows = B * net.N;
    const int ntiles = (rows + marl::kTileRows - 1) / marl::kTileRows;
    const int two = online != target;
    const size_t lds = marl::tile_lds_bytes(net.D, net.H, net.A);
    const dim3 grid((unsigned)ntiles, two ? 2u : 1u), block(marl::kThreads);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (net.H == 64)
        hipLaunchKernelGGL(marl::unroll_td_kernel<64>, grid, block, lds, stream, online->net, target->net, two, B, T,
                           obs, avail, actions, reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all);
    else
        hipLaunchKernelGGL(marl::unroll_td_kernel<128>, grid, block, lds, stream, online->net, target->net, two, B, T,
                           obs, avail, actions, reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all);
    MARL_HIP(hipGetLastError());
    return MARL_OK;
}

int marl_destroy(marl_qnet *q)
{
    if (!q) return MARL_OK;
    int rc = MARL_OK;
    {
        DeviceGuard guard(q->desc.device);
        if (q->dev_weights) {
            hipError_t err = hipFree(q->dev_weights);
            if (err != hipSuccess) rc = device_fail(err, "hipFree");
        }
    }
    delete q;
    return rc;
}

const char *marl_strerror(int status)
{
    switch (status) {
    case MARL_OK: return "ok";
    case MARL_ERR_NULL: return "a required pointer is NULL";
    case MARL_ERR_BAD_DIM: return "a size is not positive or outside the supported range";
    case MARL_ERR_BAD_DTYPE: return "unknown weight dtype";
    case MARL_ERR_MISMATCH: return "weight count or network descriptions do not match";
    case MARL_ERR_BAD_ARG: return "epsilon or gamma outside [0,1]";
    case MARL_ERR_DEVICE: return "HIP runtime error";
    case MARL_ERR_NOMEM: return "out of memory";
    default: return "unknown status";
    }
}

const char *marl_last_device_error(void) { return g_last_error; }

}  // extern "C"
