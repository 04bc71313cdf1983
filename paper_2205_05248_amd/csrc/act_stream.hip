// Streaming decision step: which networks it serves, and the dispatch to the per-shape instantiations
// (act_stream_h128.hip, act_stream_h64_bf16.hip, act_stream_h64_f32.hip; the kernel is act_stream_kernel.h).
#include "act_stream_kernel.h"

namespace marl {

hipError_t launch_act_stream_h128(const ActStreamArgs &a, int groups, hipStream_t stream);
hipError_t launch_act_stream_h64_bf16(const ActStreamArgs &a, int groups, hipStream_t stream);
hipError_t launch_act_stream_h64_f32(const ActStreamArgs &a, int groups, hipStream_t stream);

namespace {

template <int H, int P> bool stream_fits(const NetFrags &net)
{
    const int ks1 = (net.D + net.N + 31) / 32;
    if (ks1 > Stream16<H, P>::KM) return false;
    if ((64 * net.D + 1023) / 1024 > kStreamMaxObsOps * Stream16<H, P>::NW) return false;
    return StreamLds<H, P>::total(net.D) <= kLdsLimit;
}

}  // namespace

bool act_stream_fits(const NetFrags &net, int E)
{
    if (net.A > 64) return false;
    const long rows = (long)E * net.N;
    const long widest = net.D > net.H ? net.D : net.H;
    if (rows * 4 * widest >= (1l << 30)) return false;       // 32-bit byte offsets with room for the items past the end
    if (net.H == 64 && net.planes == 2) return stream_fits<64, 2>(net);
    if (net.H == 64 && net.planes == 1) return stream_fits<64, 1>(net);
    if (net.H == 128 && net.planes == 1) return stream_fits<128, 1>(net);
    return false;
}

hipError_t launch_act_stream(const NetFrags &net, int E, int n_cu, const float *obs, const uint8_t *avail,
                             const float *h_in, const uint8_t *reset, const int32_t *step_t, float epsilon,
                             uint64_t seed, float *h_out, int32_t *action, float *q_out, hipStream_t stream)
{
    ActStreamArgs a{};
    a.net = net;
    a.rows = E * net.N;
    a.n_items = (a.rows + 15) / 16;
    a.E = E;
    a.obs = obs; a.avail = avail; a.h_in = h_in; a.reset = reset; a.step_t = step_t;
    a.epsilon = epsilon; a.seed = seed; a.h_out = h_out; a.action = action; a.q_out = q_out;
    const int per_cu = net.H == 64 ? 2 : 1;                  // workgroups a compute unit holds (LDS, registers)
    const int groups = a.n_items < n_cu * per_cu ? a.n_items : n_cu * per_cu;
    if (net.H == 64 && net.planes == 2) return launch_act_stream_h64_f32(a, groups, stream);
    if (net.H == 64 && net.planes == 1) return launch_act_stream_h64_bf16(a, groups, stream);
    if (net.H == 128 && net.planes == 1) return launch_act_stream_h128(a, groups, stream);
    return hipErrorInvalidValue;
}

}  // namespace marl
