// C-ABI entry points of the recurrent Q-network library (see include/marl_qnet.h):
// argument validation, the handle, and the scratch buffer; the kernels live in kernels.hip.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "qnet_internal.h"

// Input-projection buffer of marl_unroll_td_static: device memory that exists from the moment the library is loaded
// on a device, so that the call allocates nothing.  The name stands for the array in host code only as a symbol to
// look up; the address on each device comes from static_scratch_of() below.
static __device__ __align__(256) unsigned char scratch[MARL_STATIC_SCRATCH_BYTES];

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

// The device address of `scratch` on the current device (each device holds its own copy of the array), looked up
// once per device.
constexpr int kMaxDevices = 64;
std::mutex g_static_scratch_lock;
void *g_static_scratch[kMaxDevices] = {};

int static_scratch_of(int device, void **out)
{
    if (device < 0 || device >= kMaxDevices) {
        std::snprintf(g_last_error, sizeof(g_last_error), "device %d beyond the %d devices the static scratch serves", device, kMaxDevices);
        return MARL_ERR_DEVICE;
    }
    std::lock_guard<std::mutex> hold(g_static_scratch_lock);
    if (!g_static_scratch[device]) {
        void *ptr = nullptr;
        const hipError_t err = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return device_fail(err, "hipGetSymbolAddress(scratch)");
        if (!ptr) return device_fail(hipErrorInvalidSymbol, "hipGetSymbolAddress(scratch)");
        g_static_scratch[device] = ptr;
    }
    *out = g_static_scratch[device];
    return MARL_OK;
}

bool unit_interval(float v) { return std::isfinite(v) && v >= 0.0f && v <= 1.0f; }

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Grow the handle's input-projection buffer to at least `bytes` (never shrinks).
int ensure_scratch(marl_qnet *q, size_t bytes)
{
    if (bytes <= q->scratch_bytes) return MARL_OK;
    if (q->scratch) {
        hipError_t err = hipFree(q->scratch);          // synchronises: earlier calls may still read it
        q->scratch = nullptr;
        q->scratch_bytes = 0;
        if (err != hipSuccess) return device_fail(err, "hipFree");
    }
    hipError_t err = hipMalloc(&q->scratch, bytes);
    if (err != hipSuccess) {
        q->scratch = nullptr;
        return err == hipErrorOutOfMemory ? MARL_ERR_NOMEM : device_fail(err, "hipMalloc");
    }
    q->scratch_bytes = bytes;
    return MARL_OK;
}

// Hands out `count` events for one timed call, or nullptr when the record is full.
hipEvent_t *take_events(marl_qnet *q, int count, int *rc)
{
    *rc = MARL_OK;
    if (q->timed_calls.size() >= MARL_TIMING_MAX_CALLS) return nullptr;
    while (q->ev_pool.size() < q->ev_used + count) {
        hipEvent_t e;
        hipError_t err = hipEventCreate(&e);
        if (err != hipSuccess) { *rc = device_fail(err, "hipEventCreate"); return nullptr; }
        q->ev_pool.push_back(e);
    }
    hipEvent_t *ev = &q->ev_pool[q->ev_used];
    q->ev_used += count;
    q->timed_calls.push_back(count);
    return ev;
}

// Takes back the events of the call recorded last (its launch failed).
void drop_events(marl_qnet *q, int count)
{
    q->timed_calls.pop_back();
    q->ev_used -= count;
}

}  // namespace

namespace marl {
int report_device_error(hipError_t err, const char *what) { return device_fail(err, what); }
thread_local const KernelTimer *g_kernel_timer = nullptr;
}  // namespace marl

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

    marl::PackedImage img{};
    if (!marl::pack_network(*desc, host_weights, &img)) return MARL_ERR_NOMEM;
    struct FreeHost { void *p; ~FreeHost() { std::free(p); } } free_host{img.host};

    int n_dev = 0;
    hipError_t err = hipGetDeviceCount(&n_dev);
    if (err != hipSuccess) return device_fail(err, "hipGetDeviceCount");
    if (desc->device >= n_dev) {
        std::snprintf(g_last_error, sizeof(g_last_error), "device %d not present (%d devices)", desc->device, n_dev);
        return MARL_ERR_DEVICE;
    }
    DeviceGuard guard(desc->device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");

    marl_qnet *q = new (std::nothrow) marl_qnet();
    if (!q) return MARL_ERR_NOMEM;
    q->desc = *desc;
    q->n_params = n_weights;
    q->dev_weights = nullptr;
    q->dev_weight_bytes = img.bytes;
    q->staging = nullptr;
    q->staging_done = nullptr;
    q->scratch = nullptr;
    q->scratch_bytes = 0;
    q->repack_map = nullptr;
    q->repack_elems = 0;
    q->kernels = MARL_KERNELS_AUTO;
    {
        int n_cu = 0;
        if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, desc->device) != hipSuccess || n_cu <= 0) n_cu = 256;
        q->n_cu = n_cu;
    }
    q->timing = false;
    q->ev_used = 0;
    q->static_scratch = nullptr;
    {
        const int rc = static_scratch_of(desc->device, &q->static_scratch);      // the handle's device is current here
        if (rc != MARL_OK) { delete q; return rc; }
    }
    // The backward pass's second stream (default priority) and its events are made here, not at first use: a call
    // under graph capture may create nothing.  Without them the pass runs on the caller's stream alone.
    q->side = marl::SideStream{nullptr, nullptr, nullptr};
    if (hipStreamCreateWithFlags(&q->side.stream, hipStreamNonBlocking) != hipSuccess
        || hipEventCreateWithFlags(&q->side.fork, hipEventDisableTiming) != hipSuccess
        || hipEventCreateWithFlags(&q->side.join, hipEventDisableTiming) != hipSuccess) {
        if (q->side.fork) (void)hipEventDestroy(q->side.fork);
        if (q->side.stream) (void)hipStreamDestroy(q->side.stream);
        q->side = marl::SideStream{nullptr, nullptr, nullptr};
        (void)hipGetLastError();
    }
    auto drop_side = [&]() {
        if (q->side.join) (void)hipEventDestroy(q->side.join);
        if (q->side.fork) (void)hipEventDestroy(q->side.fork);
        if (q->side.stream) (void)hipStreamDestroy(q->side.stream);
    };
    err = hipMalloc(&q->dev_weights, img.bytes);
    if (err != hipSuccess) { drop_side(); delete q; return err == hipErrorOutOfMemory ? MARL_ERR_NOMEM : device_fail(err, "hipMalloc"); }
    err = hipMemcpy(q->dev_weights, img.host, img.bytes, hipMemcpyHostToDevice);
    if (err != hipSuccess) { (void)hipFree(q->dev_weights); drop_side(); delete q; return device_fail(err, "hipMemcpy"); }

    const char *base = static_cast<const char *>(q->dev_weights);
    marl::NetFrags &n = q->net;
    n.act_stream = reinterpret_cast<const marl::bf16x8 *>(base + img.off_act);
    n.proj_stream = reinterpret_cast<const marl::bf16x8 *>(base + img.off_proj);
    n.whh = reinterpret_cast<const marl::bf16x8 *>(base + img.off_whh);
    n.w2 = reinterpret_cast<const marl::bf16x8 *>(base + img.off_w2);
    n.w1_16 = reinterpret_cast<const marl::bf16x8 *>(base + img.off_w1_16);
    n.wih_16 = reinterpret_cast<const marl::bf16x8 *>(base + img.off_wih_16);
    n.whh_16 = reinterpret_cast<const marl::bf16x8 *>(base + img.off_whh_16);
    n.w2_16 = reinterpret_cast<const marl::bf16x8 *>(base + img.off_w2_16);
    n.w1x_16 = reinterpret_cast<const marl::bf16x8 *>(base + img.off_w1x_16);
    n.wihT_16 = reinterpret_cast<const marl::bf16x8 *>(base + img.off_wihT_16);
    n.whhT_16 = reinterpret_cast<const marl::bf16x8 *>(base + img.off_whhT_16);
    n.w2_plain = reinterpret_cast<const float *>(base + img.off_w2_plain);
    n.bias1 = reinterpret_cast<const float *>(base + img.off_bias1);
    n.b1_plain = reinterpret_cast<const float *>(base + img.off_b1_plain);
    n.bias_r = reinterpret_cast<const float *>(base + img.off_bias_r);
    n.bias_z = reinterpret_cast<const float *>(base + img.off_bias_z);
    n.bias_in = reinterpret_cast<const float *>(base + img.off_bias_in);
    n.bias_hn = reinterpret_cast<const float *>(base + img.off_bias_hn);
    n.b2 = reinterpret_cast<const float *>(base + img.off_b2);
    n.N = desc->n_agents; n.D = desc->obs_dim; n.A = desc->n_actions; n.H = desc->hidden;
    n.kc1 = img.kc1; n.mb2 = img.mb2; n.planes = img.planes;
    n.nc1 = img.nc1; n.act_chunks = img.act_chunks; n.proj_chunks = img.proj_chunks;
    *out = q;
    return MARL_OK;
}

int marl_qnet_set_weights(marl_qnet *q, const float *host_weights, size_t n_weights, void *hip_stream)
{
    if (!q || !host_weights) return MARL_ERR_NULL;
    if (n_weights != q->n_params) return MARL_ERR_MISMATCH;
    marl::PackedImage img{};
    if (!marl::pack_network(q->desc, host_weights, &img)) return MARL_ERR_NOMEM;
    struct FreeHost { void *p; ~FreeHost() { std::free(p); } } free_host{img.host};
    if (img.bytes != q->dev_weight_bytes) return MARL_ERR_MISMATCH;       // cannot happen: the layout depends on the descriptor only

    DeviceGuard guard(q->desc.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    if (!q->staging) {
        hipError_t err = hipHostMalloc(&q->staging, img.bytes, hipHostMallocDefault);
        if (err != hipSuccess) { q->staging = nullptr; return err == hipErrorOutOfMemory ? MARL_ERR_NOMEM : device_fail(err, "hipHostMalloc"); }
        err = hipEventCreateWithFlags(&q->staging_done, hipEventDisableTiming);
        if (err != hipSuccess) { (void)hipHostFree(q->staging); q->staging = nullptr; q->staging_done = nullptr; return device_fail(err, "hipEventCreate"); }
    } else {
        MARL_HIP(hipEventSynchronize(q->staging_done));                   // the previous upload still reads the buffer
    }
    std::memcpy(q->staging, img.host, img.bytes);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    MARL_HIP(hipMemcpyAsync(q->dev_weights, q->staging, img.bytes, hipMemcpyHostToDevice, stream));
    MARL_HIP(hipEventRecord(q->staging_done, stream));
    return MARL_OK;
}

int marl_qnet_get_desc(const marl_qnet *q, marl_qnet_desc *out)
{
    if (!q || !out) return MARL_ERR_NULL;
    *out = q->desc;
    return MARL_OK;
}

namespace {
// AUTO: the fused kernels wherever the network fits them (they were the faster ones on every shape measured).
bool takes_fused_path(const marl_qnet *q, bool for_unroll)
{
    if (q->kernels == MARL_KERNELS_TILE32) return false;
    return for_unroll ? marl::unroll_fused_fits(q->net) : marl::act_fused_fits(q->net);
}
// The streaming decision step: on request only (slower than fused16 on every workload measured), when the
// network and the batch fit it.
bool takes_stream_path(const marl_qnet *q, int E)
{
    if (q->kernels != MARL_KERNELS_STREAM16) return false;
    return marl::act_stream_fits(q->net, E);
}
}  // namespace

int marl_act_step(marl_qnet *q, int32_t E, const float *obs, const uint8_t *avail, const float *h_in,
                  const uint8_t *reset, const int32_t *step_t, float epsilon, uint64_t seed,
                  float *h_out, int32_t *action, float *q_out, void *hip_stream)
{
    if (!q) return MARL_ERR_NULL;
    if (E < 0 || (int64_t)E * q->desc.n_agents >= (int64_t)1 << 30) return MARL_ERR_BAD_DIM;
    if (!unit_interval(epsilon)) return MARL_ERR_BAD_ARG;
    if (E == 0) return MARL_OK;
    if (!obs || !avail || !h_in || !step_t || !h_out || !action) return MARL_ERR_NULL;
    if (!aligned16(h_in) || !aligned16(h_out)) return MARL_ERR_BAD_ARG;

    DeviceGuard guard(q->desc.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const bool all_aligned = aligned16(obs) && aligned16(avail) && aligned16(step_t) && (!q_out || aligned16(q_out)) && aligned16(action);
    const bool stream_path = takes_stream_path(q, E) && all_aligned;
    const bool fused_path = takes_fused_path(q, false) && marl::act_fused_rows_fit(q->net, E);
    hipEvent_t *ev = nullptr;
    if (q->timing) {
        q->ev_pool.reserve(3 * MARL_TIMING_MAX_CALLS);      // keeps handed-out pointers stable
        int rc;
        ev = take_events(q, 2, &rc);
        if (rc != MARL_OK) return rc;
    }
    // one-kernel paths: the events take the kernel's own start and end; the tile32 path records them around its launches
    marl::KernelTimer timer{};
    if (ev && (stream_path || fused_path)) {
        timer = {ev[0], ev[1]};
        marl::g_kernel_timer = &timer;
    }
    hipError_t err = hipSuccess;
    if (stream_path) {
        err = marl::launch_act_stream(q->net, E, q->n_cu, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action, q_out, stream);
    } else if (fused_path) {
        err = marl::launch_act_fused(q->net, E, nullptr, 0, q->n_cu, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action, q_out, stream);
    } else {
        if (ev) err = hipEventRecord(ev[0], stream);
        if (err == hipSuccess) err = marl::launch_act_step(q->net, E, nullptr, 0, obs, avail, h_in, reset, step_t, epsilon, seed, h_out, action, q_out, stream);
        if (err == hipSuccess && ev) err = hipEventRecord(ev[1], stream);
    }
    marl::g_kernel_timer = nullptr;
    if (err != hipSuccess) {
        if (ev) drop_events(q, 2);                         // the record must not keep events that were never recorded
        return device_fail(err, "marl_act_step launch");
    }
    return MARL_OK;
}

int marl_act_step_indexed(marl_qnet *q, int32_t E, const int32_t *env_index, int32_t n_listed, const float *obs,
                          const uint8_t *avail, const float *h_in, const uint8_t *reset, const int32_t *step_t,
                          float epsilon, uint64_t seed, float *h_out, int32_t *action, float *q_out, void *hip_stream)
{
    if (!q) return MARL_ERR_NULL;
    if (E < 0 || (int64_t)E * q->desc.n_agents >= (int64_t)1 << 30 || n_listed < 0 || n_listed > E) return MARL_ERR_BAD_DIM;
    if (!unit_interval(epsilon)) return MARL_ERR_BAD_ARG;
    if (n_listed == 0) return MARL_OK;
    if (!env_index || !obs || !avail || !h_in || !step_t || !h_out || !action) return MARL_ERR_NULL;
    if (!aligned16(h_in) || !aligned16(h_out)) return MARL_ERR_BAD_ARG;
    DeviceGuard guard(q->desc.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // the fused kernel where the network and the arrays fit it (the tiled one on request or otherwise)
    if (takes_fused_path(q, false) && marl::act_fused_indexed_fits(q->net, E) && (!q_out || aligned16(q_out)))
        MARL_HIP(marl::launch_act_fused(q->net, E, env_index, n_listed, q->n_cu, obs, avail, h_in, reset, step_t, epsilon, seed,
                                        h_out, action, q_out, stream));
    else
        MARL_HIP(marl::launch_act_step(q->net, E, env_index, n_listed, obs, avail, h_in, reset, step_t, epsilon, seed, h_out,
                                       action, q_out, stream));
    return MARL_OK;
}

int marl_qnet_reserve_unroll(marl_qnet *q, int32_t B, int32_t T)
{
    if (!q) return MARL_ERR_NULL;
    if (B < 0 || T < 1 || (int64_t)B * q->desc.n_agents >= (int64_t)1 << 30 || (int64_t)T > (int64_t)1 << 20)
        return MARL_ERR_BAD_DIM;
    DeviceGuard guard(q->desc.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    if (takes_fused_path(q, true)) return MARL_OK;
    return ensure_scratch(q, marl::unroll_scratch_bytes(q->net, B, T));
}

int marl_qnet_kernels_in_use(const marl_qnet *q, int32_t entry)
{
    if (!q) return MARL_ERR_NULL;
    if (entry != MARL_ENTRY_ACT_STEP && entry != MARL_ENTRY_UNROLL_TD) return MARL_ERR_BAD_ARG;
    if (entry == MARL_ENTRY_ACT_STEP && takes_stream_path(q, 1)) return MARL_KERNELS_STREAM16;
    return takes_fused_path(q, entry == MARL_ENTRY_UNROLL_TD) ? MARL_KERNELS_FUSED16 : MARL_KERNELS_TILE32;
}

int marl_qnet_set_kernels(marl_qnet *q, int32_t path)
{
    if (!q) return MARL_ERR_NULL;
    if (path != MARL_KERNELS_AUTO && path != MARL_KERNELS_TILE32 && path != MARL_KERNELS_FUSED16 && path != MARL_KERNELS_STREAM16) return MARL_ERR_BAD_ARG;
    if (path == MARL_KERNELS_FUSED16 && !(marl::unroll_fused_fits(q->net) && marl::act_fused_fits(q->net))) return MARL_ERR_BAD_DIM;
    if (path == MARL_KERNELS_STREAM16 && !(marl::unroll_fused_fits(q->net) && marl::act_stream_fits(q->net, 1))) return MARL_ERR_BAD_DIM;
    q->kernels = path;
    return MARL_OK;
}

}  // extern "C"

namespace {
int unroll_call(marl_qnet *online, marl_qnet *target, int32_t B, int32_t T, const int32_t *episode_index,
                int32_t pool_episodes, const float *obs, const uint8_t *avail, const int32_t *actions,
                const float *reward, const uint8_t *terminated, const uint8_t *filled, float gamma, float *q_taken,
                float *next_max, float *td_target, float *q_all, void *hip_stream, bool double_q = false,
                int32_t *next_action = nullptr, void *keep_workspace = nullptr, bool no_alloc = false)
{
    if (no_alloc) g_last_error[0] = '\0';                // whatever this call leaves there is its own
    if (!online || !target) return MARL_ERR_NULL;
    const marl_qnet_desc &a = online->desc, &b = target->desc;
    if (a.n_agents != b.n_agents || a.obs_dim != b.obs_dim || a.n_actions != b.n_actions || a.hidden != b.hidden ||
        a.weight_dtype != b.weight_dtype || a.device != b.device)
        return MARL_ERR_MISMATCH;
    if (B < 0 || T < 1 || (int64_t)T > (int64_t)1 << 20) return MARL_ERR_BAD_DIM;
    {   // every array is indexed with 32-bit element offsets
        const int64_t widest = a.obs_dim > a.n_actions ? a.obs_dim : a.n_actions;
        const int64_t episodes = episode_index ? (pool_episodes > B ? pool_episodes : B) : B;
        if (episodes * (T + 1) * a.n_agents * widest >= (int64_t)1 << 30) return MARL_ERR_BAD_DIM;
    }
    if (!unit_interval(gamma)) return MARL_ERR_BAD_ARG;
    if (episode_index && pool_episodes < 1) return MARL_ERR_BAD_DIM;
    if (B == 0) return MARL_OK;
    if (!obs || !avail || !actions || !reward || !terminated || !filled || !q_taken || !next_max || !td_target)
        return MARL_ERR_NULL;
    if (double_q && !next_action) return MARL_ERR_NULL;

    DeviceGuard guard(a.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    const bool two = online != target && !double_q;      // the double-estimator target runs the networks one after the other
    // no_alloc: the tiled kernels, with both networks' projections in the device's static array
    const bool fused = !no_alloc && takes_fused_path(online, true);
    int rc = MARL_OK;
    void *scratch_on = nullptr, *scratch_tg = nullptr;
    if (no_alloc) {
        const size_t need = (marl::unroll_scratch_bytes(online->net, B, T) + 255) & ~(size_t)255;
        const size_t total = online != target ? 2 * need : need;
        if (total > (size_t)MARL_STATIC_SCRATCH_BYTES) {
            std::snprintf(g_last_error, sizeof(g_last_error),
                          "marl_unroll_td_static: B = %d, T = %d needs %zu bytes of scratch, the static buffer holds %zu", B, T,
                          total, (size_t)MARL_STATIC_SCRATCH_BYTES);
            return MARL_ERR_BAD_DIM;
        }
        scratch_on = online->static_scratch;
        scratch_tg = online != target ? static_cast<char *>(online->static_scratch) + need : scratch_on;
    } else if (!fused) {
        const size_t need = marl::unroll_scratch_bytes(online->net, B, T);
        rc = ensure_scratch(online, need);
        if (rc == MARL_OK && online != target) rc = ensure_scratch(target, need);
        if (rc != MARL_OK) return rc;
        scratch_on = online->scratch;
        scratch_tg = target->scratch;
    }
    if (keep_workspace && !fused) return MARL_ERR_BAD_DIM;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    hipEvent_t *ev = nullptr;
    if (online->timing && !no_alloc) {                    // (creating events allocates)
        online->ev_pool.reserve(3 * MARL_TIMING_MAX_CALLS);
        ev = take_events(online, 3, &rc);
        if (rc != MARL_OK) return rc;
    }
    // Events of a timed call: [0] before anything, [1] between the input projection and the recurrence (tile32) or the
    // start of the last kernel (fused16: its own start, by an extended launch), [2] the end.
    marl::KernelTimer timer{};
    auto time_next_kernel = [&]() {
        if (!ev) return;
        timer = {ev[1], ev[2]};
        marl::g_kernel_timer = &timer;
    };
    auto run = [&]() -> hipError_t {
        hipError_t err = hipSuccess;
        if (ev) err = hipEventRecord(ev[0], stream);
        if (err != hipSuccess) return err;
        if (double_q) {
            // Selection by the online network (q_taken, q_all, next_action), then valuation by the target
            // network (next_max, td_target); the stream orders the second launch after the first.
            if (fused) {
                err = marl::launch_unroll_fused(online->net, online->net, false, B, T, episode_index, pool_episodes, obs,
                                                avail, actions, reward, terminated, filled, gamma, q_taken, nullptr,
                                                nullptr, q_all, stream, marl::kTdSelect, next_action);
                if (err != hipSuccess) return err;
                time_next_kernel();
                return marl::launch_unroll_fused(target->net, target->net, false, B, T, episode_index, pool_episodes, obs,
                                                 avail, actions, reward, terminated, filled, gamma, nullptr, next_max,
                                                 td_target, nullptr, stream, marl::kTdValue, next_action);
            }
            err = marl::launch_unroll_td(online->net, online->net, false, scratch_on, scratch_on, B, T,
                                         episode_index, pool_episodes, obs, avail, actions, reward, terminated,
                                         filled, gamma, q_taken, nullptr, nullptr, q_all, stream,
                                         ev ? ev[1] : nullptr, marl::kTdSelect, next_action);
            if (err != hipSuccess) return err;
            err = marl::launch_unroll_td(target->net, target->net, false, scratch_tg, scratch_tg, B, T,
                                         episode_index, pool_episodes, obs, avail, actions, reward, terminated,
                                         filled, gamma, nullptr, next_max, td_target, nullptr, stream, nullptr,
                                         marl::kTdValue, next_action);
            if (err == hipSuccess && ev) err = hipEventRecord(ev[2], stream);
            return err;
        }
        if (keep_workspace) {
            float *h_all;
            void *x_all;
            marl::qnet_grad_activation_slots(online->net, B, T, keep_workspace, &h_all, &x_all);
            time_next_kernel();
            return marl::launch_unroll_fused(online->net, target->net, two, B, T, episode_index, pool_episodes, obs, avail, actions,
                                             reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all, stream,
                                             marl::kTdKeep, nullptr, h_all, x_all);
        }
        if (fused) {
            time_next_kernel();
            return marl::launch_unroll_fused(online->net, target->net, two, B, T, episode_index, pool_episodes, obs, avail, actions, reward, terminated,
                                             filled, gamma, q_taken, next_max, td_target, q_all, stream);
        }
        err = marl::launch_unroll_td(online->net, target->net, two, scratch_on, scratch_tg, B, T, episode_index,
                                     pool_episodes, obs, avail,
                                     actions, reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all,
                                     stream, ev ? ev[1] : nullptr);
        if (err == hipSuccess && ev) err = hipEventRecord(ev[2], stream);
        return err;
    };
    const hipError_t err = run();
    marl::g_kernel_timer = nullptr;
    if (err != hipSuccess) {
        if (ev) drop_events(online, 3);                    // the record must not keep events that were never recorded
        return device_fail(err, "unroll launch");
    }
    return MARL_OK;
}
}  // namespace

extern "C" {

int marl_unroll_td(marl_qnet *online, marl_qnet *target, int32_t B, int32_t T, const float *obs,
                   const uint8_t *avail, const int32_t *actions, const float *reward, const uint8_t *terminated,
                   const uint8_t *filled, float gamma, float *q_taken, float *next_max, float *td_target,
                   float *q_all, void *hip_stream)
{
    return unroll_call(online, target, B, T, nullptr, B, obs, avail, actions, reward, terminated, filled, gamma,
                       q_taken, next_max, td_target, q_all, hip_stream);
}

int marl_unroll_td_static(marl_qnet *online, marl_qnet *target, int32_t B, int32_t T, const float *obs,
                          const uint8_t *avail, const int32_t *actions, const float *reward, const uint8_t *terminated,
                          const uint8_t *filled, float gamma, float *q_taken, float *next_max, float *td_target,
                          float *q_all, void *hip_stream)
{
    return unroll_call(online, target, B, T, nullptr, B, obs, avail, actions, reward, terminated, filled, gamma,
                       q_taken, next_max, td_target, q_all, hip_stream, false, nullptr, nullptr, true);
}

int marl_unroll_td_indexed(marl_qnet *online, marl_qnet *target, int32_t pool_episodes, const int32_t *episode_index,
                           int32_t B, int32_t T, const float *obs, const uint8_t *avail, const int32_t *actions,
                           const float *reward, const uint8_t *terminated, const uint8_t *filled, float gamma,
                           float *q_taken, float *next_max, float *td_target, float *q_all, void *hip_stream)
{
    if (B > 0 && !episode_index) return MARL_ERR_NULL;
    return unroll_call(online, target, B, T, episode_index, pool_episodes, obs, avail, actions, reward, terminated,
                       filled, gamma, q_taken, next_max, td_target, q_all, hip_stream);
}

int marl_unroll_td_double(marl_qnet *online, marl_qnet *target, int32_t pool_episodes, const int32_t *episode_index,
                          int32_t B, int32_t T, const float *obs, const uint8_t *avail, const int32_t *actions,
                          const float *reward, const uint8_t *terminated, const uint8_t *filled, float gamma,
                          float *q_taken, float *next_max, float *td_target, int32_t *next_action, float *q_all,
                          void *hip_stream)
{
    return unroll_call(online, target, B, T, episode_index, episode_index ? pool_episodes : B, obs, avail, actions,
                       reward, terminated, filled, gamma, q_taken, next_max, td_target, q_all, hip_stream, true,
                       next_action);
}

int marl_qnet_grad_workspace_bytes(const marl_qnet *q, int32_t B, int32_t T, size_t *bytes)
{
    if (!q || !bytes) return MARL_ERR_NULL;
    if (B < 1 || T < 1 || (int64_t)B * q->desc.n_agents * ((int64_t)T + 1) * 4 * q->desc.hidden >= (int64_t)1 << 30)
        return MARL_ERR_BAD_DIM;
    if (!marl::qnet_grad_fits(q->net)) return MARL_ERR_BAD_DIM;
    *bytes = marl::qnet_grad_workspace_bytes(q->net, B, T);
    return MARL_OK;
}

namespace {
int qnet_grad_call(marl_qnet *q, int32_t B, int32_t T, const float *obs, const int32_t *actions, const uint8_t *filled,
                   const float *grad_q_taken, void *workspace, size_t workspace_bytes, float *grad_weights,
                   void *hip_stream, bool activations_kept)
{
    if (!q) return MARL_ERR_NULL;
    size_t need = 0;
    const int rc = marl_qnet_grad_workspace_bytes(q, B, T, &need);
    if (rc != MARL_OK) return rc;
    {
        const marl_qnet_desc &a = q->desc;
        const int64_t widest = a.obs_dim > a.n_actions ? a.obs_dim : a.n_actions;
        if ((int64_t)B * (T + 1) * a.n_agents * widest >= (int64_t)1 << 30 || (int64_t)T > (int64_t)1 << 20) return MARL_ERR_BAD_DIM;
    }
    if (!obs || !actions || !filled || !grad_q_taken || !workspace || !grad_weights) return MARL_ERR_NULL;
    if (workspace_bytes < need) return MARL_ERR_BAD_DIM;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return MARL_ERR_BAD_ARG;
    DeviceGuard guard(q->desc.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    MARL_HIP(marl::launch_qnet_grad(q->net, B, T, obs, actions, filled, grad_q_taken, workspace, grad_weights,
                                    static_cast<hipStream_t>(hip_stream), activations_kept, &q->side, q->n_cu));
    return MARL_OK;
}
}  // namespace

int marl_qnet_grad(marl_qnet *q, int32_t B, int32_t T, const float *obs, const int32_t *actions, const uint8_t *filled,
                   const float *grad_q_taken, void *workspace, size_t workspace_bytes, float *grad_weights,
                   void *hip_stream)
{
    return qnet_grad_call(q, B, T, obs, actions, filled, grad_q_taken, workspace, workspace_bytes, grad_weights, hip_stream, false);
}

int marl_qnet_grad_kept(marl_qnet *q, int32_t B, int32_t T, const float *obs, const int32_t *actions, const uint8_t *filled,
                        const float *grad_q_taken, void *workspace, size_t workspace_bytes, float *grad_weights,
                        void *hip_stream)
{
    return qnet_grad_call(q, B, T, obs, actions, filled, grad_q_taken, workspace, workspace_bytes, grad_weights, hip_stream, true);
}

int marl_unroll_td_keep(marl_qnet *online, marl_qnet *target, int32_t B, int32_t T, const float *obs,
                        const uint8_t *avail, const int32_t *actions, const float *reward, const uint8_t *terminated,
                        const uint8_t *filled, float gamma, float *q_taken, float *next_max, float *td_target,
                        float *q_all, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    if (!online || !workspace) return MARL_ERR_NULL;
    size_t need = 0;
    const int rc = marl_qnet_grad_workspace_bytes(online, B, T, &need);
    if (rc != MARL_OK) return rc;
    if (workspace_bytes < need) return MARL_ERR_BAD_DIM;
    if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return MARL_ERR_BAD_ARG;
    return unroll_call(online, target, B, T, nullptr, B, obs, avail, actions, reward, terminated, filled, gamma, q_taken,
                       next_max, td_target, q_all, hip_stream, false, nullptr, workspace);
}

int marl_qnet_check_refresh_map(const marl_qnet_desc *desc, const float *host_weights, size_t n_weights)
{
    if (!desc || !host_weights) return MARL_ERR_NULL;
    int why;
    if (!desc_valid(desc, &why)) return why;
    if (n_weights != param_count(desc)) return MARL_ERR_MISMATCH;
    return marl::repack_map_reproduces_packer(*desc, host_weights, n_weights) ? MARL_OK : MARL_ERR_MISMATCH;
}

namespace {
bool is_finite(float v) { return v == v && v - v == 0.0f; }

int qnet_update(marl_qnet *q, float *weights, const float *grad_weights, float lr, const marl::UpdateRule &rule, void *hip_stream)
{
    DeviceGuard guard(q->desc.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    if (!q->repack_map) {
        std::vector<int32_t> map;
        if (!marl::build_repack_map(q->desc, q->n_params, &map, &q->layout)) return MARL_ERR_NOMEM;
        int32_t *dev = nullptr;
        hipError_t err = hipMalloc(&dev, map.size() * sizeof(int32_t));
        if (err != hipSuccess) return err == hipErrorOutOfMemory ? MARL_ERR_NOMEM : device_fail(err, "hipMalloc");
        err = hipMemcpy(dev, map.data(), map.size() * sizeof(int32_t), hipMemcpyHostToDevice);
        if (err != hipSuccess) { (void)hipFree(dev); return device_fail(err, "hipMemcpy"); }
        q->repack_map = dev;
        q->repack_elems = map.size();
    }
    MARL_HIP(marl::launch_sgd_step(q->desc, q->layout, q->net.planes, q->repack_map, q->repack_elems, q->dev_weights, weights,
                                   grad_weights, q->n_params, lr, static_cast<hipStream_t>(hip_stream), rule));
    return MARL_OK;
}
}  // namespace

int marl_qnet_sgd_step(marl_qnet *q, float *weights, const float *grad_weights, float lr, void *hip_stream)
{
    if (!q || !weights || !grad_weights) return MARL_ERR_NULL;
    if (!is_finite(lr)) return MARL_ERR_BAD_ARG;
    return qnet_update(q, weights, grad_weights, lr, marl::UpdateRule(), hip_stream);
}

int marl_qnet_rmsprop_step(marl_qnet *q, float *weights, const float *grad_weights, float *sq_avg, float lr, float alpha,
                           float eps, void *hip_stream)
{
    if (!q || !weights || !grad_weights || !sq_avg) return MARL_ERR_NULL;
    if (!is_finite(lr) || !(alpha >= 0.0f && alpha <= 1.0f) || !(eps > 0.0f) || !is_finite(eps)) return MARL_ERR_BAD_ARG;
    marl::UpdateRule rule;
    rule.sq_avg = sq_avg; rule.alpha = alpha; rule.eps = eps;
    return qnet_update(q, weights, grad_weights, lr, rule, hip_stream);
}

int marl_qnet_set_timing(marl_qnet *q, int32_t enable)
{
    if (!q) return MARL_ERR_NULL;
    q->timing = enable != 0;
    q->ev_used = 0;
    q->timed_calls.clear();
    return MARL_OK;
}

int marl_qnet_timing_read(marl_qnet *q, float *act_ms, int32_t *act_calls, float unroll_ms[2], int32_t *unroll_calls)
{
    if (!q || !act_ms || !act_calls || !unroll_ms || !unroll_calls) return MARL_ERR_NULL;
    DeviceGuard guard(q->desc.device);
    if (!guard.ok) return device_fail(hipErrorInvalidDevice, "hipSetDevice");
    double act = 0.0, proj = 0.0, rec = 0.0;
    int n_act = 0, n_unroll = 0;
    size_t at = 0;
    hipError_t err = hipSuccess;
    for (int count : q->timed_calls) {
        hipEvent_t *ev = &q->ev_pool[at];
        at += count;
        float a = 0.0f, b = 0.0f;
        err = hipEventSynchronize(ev[count - 1]);
        if (err == hipSuccess) err = hipEventElapsedTime(&a, ev[0], ev[1]);
        if (err == hipSuccess && count == 3) err = hipEventElapsedTime(&b, ev[1], ev[2]);
        if (err != hipSuccess) break;
        if (count == 2) { act += a; ++n_act; continue; }
        proj += a; rec += b; ++n_unroll;
    }
    if (err != hipSuccess) {                               // the record is cleared either way: a later read starts afresh
        q->ev_used = 0;
        q->timed_calls.clear();
        return device_fail(err, "marl_qnet_timing_read");
    }
    *act_ms = n_act ? (float)(act / n_act) : 0.0f;
    *act_calls = n_act;
    unroll_ms[0] = n_unroll ? (float)(proj / n_unroll) : 0.0f;
    unroll_ms[1] = n_unroll ? (float)(rec / n_unroll) : 0.0f;
    *unroll_calls = n_unroll;
    q->ev_used = 0;
    q->timed_calls.clear();
    return MARL_OK;
}

int marl_destroy(marl_qnet *q)
{
    if (!q) return MARL_OK;
    int rc = MARL_OK;
    {
        DeviceGuard guard(q->desc.device);
        for (hipEvent_t e : q->ev_pool) (void)hipEventDestroy(e);
        for (void *p : {q->dev_weights, q->scratch, static_cast<void *>(q->repack_map)}) {
            if (!p) continue;
            hipError_t err = hipFree(p);
            if (err != hipSuccess) rc = device_fail(err, "hipFree");        // hipFree waits for the device
        }
        if (q->staging_done) (void)hipEventDestroy(q->staging_done);
        if (q->staging) (void)hipHostFree(q->staging);
        if (q->side.join) (void)hipEventDestroy(q->side.join);
        if (q->side.fork) (void)hipEventDestroy(q->side.fork);
        if (q->side.stream) (void)hipStreamDestroy(q->side.stream);
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
