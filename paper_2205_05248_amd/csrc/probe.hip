// Measurement aids: what this GPU reaches on two plain kernels, to set next to the nominal peaks in a benchmark.
// Neither is part of the recurrent network's path.
#include <hip/hip_runtime.h>

#include "qnet_internal.h"

namespace {

typedef float f32x4_t __attribute__((ext_vector_type(4)));

// Every workgroup walks the buffer with the whole grid's stride, four 16-byte vectors per lane in flight.
template <bool COPY>
__global__ __launch_bounds__(256) void stream_probe_kernel(const f32x4_t *__restrict__ src, f32x4_t *__restrict__ dst,
                                                           size_t n_vec, float *__restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    f32x4_t acc = {0.0f, 0.0f, 0.0f, 0.0f};
    for (; i + 3 * stride < n_vec; i += 4 * stride) {
        f32x4_t v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = __builtin_nontemporal_load(src + i + j * stride);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if constexpr (COPY) __builtin_nontemporal_store(v[j], dst + i + j * stride);
            else acc += v[j];
        }
    }
    for (; i < n_vec; i += stride) {
        const f32x4_t v = __builtin_nontemporal_load(src + i);
        if constexpr (COPY) __builtin_nontemporal_store(v, dst + i);
        else acc += v;
    }
    if constexpr (!COPY) {
        // keeps the loads alive; the store itself almost never happens
        if (acc[0] + acc[1] + acc[2] + acc[3] == 1.2345e38f) sink[0] = acc[0];
    }
}

// Four waves per workgroup, eight independent accumulators per wave: the matrix pipe never waits on a dependency.
__global__ __launch_bounds__(256) void mfma_probe_kernel(int iters, float *__restrict__ sink)
{
    marl::bf16x8 a, b;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
    }
    f32x4_t acc[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) acc[k] = {0.0f, 0.0f, 0.0f, 0.0f};
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int k = 0; k < 8; ++k) acc[k] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[k], 0, 0, 0);
    }
    float total = 0.0f;
#pragma unroll
    for (int k = 0; k < 8; ++k) total += acc[k][0] + acc[k][1] + acc[k][2] + acc[k][3];
    if (total == -1.0f) sink[0] = total;                  // sums of non-negative products: never
}

int cu_count()
{
    int dev = 0, n_cu = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0) return 256;
    return n_cu;
}

}  // namespace

extern "C" {

int marl_probe_stream(const void *src, void *dst, size_t bytes, float *sink, void *hip_stream)
{
    if (!src || !sink) return MARL_ERR_NULL;
    if (bytes == 0 || bytes % 16 != 0) return MARL_ERR_BAD_DIM;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return MARL_ERR_BAD_ARG;
    const size_t n_vec = bytes / 16;
    const dim3 grid((unsigned)(cu_count() * 32)), block(256);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (dst)
        hipLaunchKernelGGL(stream_probe_kernel<true>, grid, block, 0, stream, static_cast<const f32x4_t *>(src),
                           static_cast<f32x4_t *>(dst), n_vec, sink);
    else
        hipLaunchKernelGGL(stream_probe_kernel<false>, grid, block, 0, stream, static_cast<const f32x4_t *>(src),
                           static_cast<f32x4_t *>(nullptr), n_vec, sink);
    const hipError_t err = hipGetLastError();
    return err == hipSuccess ? MARL_OK : marl::report_device_error(err, "probe launch");
}

int marl_probe_mfma(int32_t iters, float *sink, double *flops, void *hip_stream)
{
    if (!sink || !flops) return MARL_ERR_NULL;
    if (iters < 1 || iters > (1 << 24)) return MARL_ERR_BAD_DIM;
    const int groups = cu_count() * 2;                    // two waves on every SIMD
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)groups), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters, sink);
    const hipError_t err = hipGetLastError();
    if (err != hipSuccess) return marl::report_device_error(err, "probe launch");
    *flops = (double)groups * 4 * (double)iters * 8 * (2.0 * 16 * 16 * 32);
    return MARL_OK;
}

}  // extern "C"
