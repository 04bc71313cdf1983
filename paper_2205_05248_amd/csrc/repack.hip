// The learner's parameter update on the device (Alg. 3, last step of the loop): the packed fp32 weights move
// by -lr * gradient, and the image the kernels read (MFMA operand fragments, bias tables) is rebuilt from
// them in place, stream-ordered, without a trip through the host.
//
// The fragment part of the image is a permutation of the parameters with some positions left zero; every
// 16-bit element holds either the bf16 nearest to one parameter or the bf16 of what that rounding left over.
// Which parameter, and which of the two, is found once per handle by asking the host packer itself: it is
// run on three weight vectors whose entries spell the digits of their own index in base 128, each digit d
// written as (d + 1) (1 + 2^-9), a value whose bf16 rounding is d + 1 and whose remainder is (d + 1) 2^-9,
// so both planes of the result can be read back.  The device kernel then applies that map to any weights
// with the packer's own rounding.  The fp32 tables at the end of the image are few and are written out.
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>

#include <vector>

#include "qnet_internal.h"

namespace marl {
namespace {

constexpr int32_t kNoSource = -1;
constexpr int32_t kLowPlane = 1 << 30;        // map entry: parameter index, + this bit for the remainder plane

float bf16_to_float(uint16_t bits)
{
    const uint32_t b = (uint32_t)bits << 16;
    float v;
    std::memcpy(&v, &b, 4);
    return v;
}

// bits of the bf16 nearest to v, ties to even (no NaN handling: weights are finite)
__device__ __forceinline__ uint32_t bf16_rne(float v)
{
    uint32_t b = __float_as_uint(v);
    b += 0x7FFFu + ((b >> 16) & 1u);
    return b >> 16;
}

__global__ void sgd_kernel(float *w, const float *g, float lr, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        float step = lr * g[i];
        asm volatile("" : "+v"(step));           // the product is rounded on its own: no fused multiply-add
        w[i] = w[i] - step;
    }
}

// RMSprop: v <- alpha v + (1 - alpha) g^2;  w <- w - lr g / (sqrt(v) + eps).  Every operation is rounded on its
// own, in this order (no fused multiply-add), so that a host reference in fp32 reproduces it bit for bit.
__global__ void rmsprop_kernel(float *w, const float *g, float *v, float lr, float alpha, float eps, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float gi = g[i];
    float keep = alpha * v[i];
    asm volatile("" : "+v"(keep));
    float sq = gi * gi;
    asm volatile("" : "+v"(sq));
    float fresh = (1.0f - alpha) * sq;
    asm volatile("" : "+v"(fresh));
    const float vi = keep + fresh;
    v[i] = vi;
    const float denom = sqrtf(vi) + eps;          // sqrtf and / are correctly rounded (the compiler's default for HIP)
    float ratio = gi / denom;
    asm volatile("" : "+v"(ratio));
    float step = lr * ratio;
    asm volatile("" : "+v"(step));
    w[i] = w[i] - step;
}

__device__ __forceinline__ void repack_frag_element(const float *w, const int32_t *map, uint16_t *image, size_t n, size_t e)
{
    if (e >= n) return;
    const int32_t m = map[e];
    uint32_t out = 0;
    if (m != kNoSource) {
        const float v = w[m & (kLowPlane - 1)];
        const uint32_t hi = bf16_rne(v);
        out = (m & kLowPlane) ? bf16_rne(__fsub_rn(v, __uint_as_float(hi << 16))) : hi;
    }
    image[e] = (uint16_t)out;
}

__global__ void repack_frag_kernel(const float *w, const int32_t *map, uint16_t *image, size_t n)
{
    repack_frag_element(w, map, image, n, (size_t)blockIdx.x * blockDim.x + threadIdx.x);
}

// fp32 tables that are plain copies of parameters: dst[i] = w[src[i]]
__global__ void copy_map_kernel(const float *w, const int32_t *src, float *dst, size_t n)
{
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) dst[i] = w[src[i]];
}

struct TableArgs {
    const float *w;
    char *image;
    size_t off_w2_plain, off_bias1, off_b1_plain, off_bias_r, off_bias_z, off_bias_in, off_bias_hn, off_b2;
    int N, D, A, H, planes;
};

__device__ __forceinline__ void repack_table_entries(const TableArgs &t, int i)
{
    const int N = t.N, D = t.D, A = t.A, H = t.H, Din = D + N;
    const float *W1 = t.w, *b1 = W1 + (size_t)H * Din, *Wih = b1 + H, *Whh = Wih + (size_t)3 * H * H;
    const float *bih = Whh + (size_t)3 * H * H, *bhh = bih + 3 * H, *W2 = bhh + 3 * H, *b2 = W2 + (size_t)A * H;
    auto as_stored = [&](float v) { return t.planes == 1 ? __uint_as_float(bf16_rne(v) << 16) : v; };
    if (i < A * H) reinterpret_cast<float *>(t.image + t.off_w2_plain)[i] = as_stored(W2[i]);
    if (i < N * H) {
        const int n = i / H, j = i % H;
        reinterpret_cast<float *>(t.image + t.off_bias1)[i] = __fadd_rn(b1[j], as_stored(W1[(size_t)j * Din + D + n]));
    }
    if (i < H) {
        reinterpret_cast<float *>(t.image + t.off_b1_plain)[i] = b1[i];
        reinterpret_cast<float *>(t.image + t.off_bias_r)[i] = __fadd_rn(bih[i], bhh[i]);
        reinterpret_cast<float *>(t.image + t.off_bias_z)[i] = __fadd_rn(bih[H + i], bhh[H + i]);
        reinterpret_cast<float *>(t.image + t.off_bias_in)[i] = bih[2 * H + i];
        reinterpret_cast<float *>(t.image + t.off_bias_hn)[i] = bhh[2 * H + i];
    }
    if (i < A) reinterpret_cast<float *>(t.image + t.off_b2)[i] = b2[i];
}

// The whole image of a Q-network from its updated weights in one launch: the first frag_blocks workgroups rebuild
// the fragment part, the others the fp32 tables (the two do not depend on each other).
__global__ void repack_image_kernel(const float *w, const int32_t *map, uint16_t *image, size_t n, unsigned frag_blocks, TableArgs t)
{
    if (blockIdx.x < frag_blocks) repack_frag_element(w, map, image, n, (size_t)blockIdx.x * blockDim.x + threadIdx.x);
    else repack_table_entries(t, (int)((blockIdx.x - frag_blocks) * blockDim.x + threadIdx.x));
}

}  // namespace

// Host: map[e] for every 16-bit element e of an image's fragment part, found by running its packer on the probe
// vectors described at the top of this file.  pack(w, out) writes the frag_elems elements packed from w.
bool probe_fragment_map(size_t n_params, size_t frag_elems, const FragPacker &pack, std::vector<int32_t> *map)
{
    if (n_params >= (size_t)128 * 128 * 128) return false;
    std::vector<float> probe(n_params);
    std::vector<uint16_t> images[3];
    for (int k = 0; k < 3; ++k) {
        for (size_t i = 0; i < n_params; ++i) {
            const int digit = (int)((i >> (7 * k)) & 127);
            probe[i] = (float)(digit + 1) * (1.0f + 1.0f / 512.0f);
        }
        images[k].assign(frag_elems, 0);
        if (!pack(probe.data(), images[k].data())) return false;
    }
    map->assign(frag_elems, kNoSource);
    for (size_t e = 0; e < frag_elems; ++e) {
        if (!images[0][e] && !images[1][e] && !images[2][e]) continue;
        int32_t index = 0, plane = -1;
        for (int k = 0; k < 3; ++k) {
            const float v = bf16_to_float(images[k][e]);
            const int this_plane = v >= 1.0f ? 0 : 1;
            const float scaled = this_plane ? v * 512.0f : v;
            const int digit = (int)std::lround(scaled) - 1;
            if (digit < 0 || digit > 127 || (float)(digit + 1) != scaled || (plane >= 0 && plane != this_plane)) return false;
            plane = this_plane;
            index |= digit << (7 * k);
        }
        if ((size_t)index >= n_params) return false;
        (*map)[e] = index | (plane ? kLowPlane : 0);
    }
    return true;
}

// The Q-network's image: fragments in bytes [0, off_w2_plain); also returns the image's layout.
bool build_repack_map(const marl_qnet_desc &desc, size_t n_params, std::vector<int32_t> *map, PackedImage *layout)
{
    std::vector<float> zeros(n_params, 0.0f);
    PackedImage first{};
    if (!pack_network(desc, zeros.data(), &first)) return false;
    std::free(first.host);
    *layout = first;
    layout->host = nullptr;
    const size_t elems = first.off_w2_plain / 2;
    return probe_fragment_map(n_params, elems, [&](const float *w, uint16_t *out) {
        PackedImage img{};
        if (!pack_network(desc, w, &img)) return false;
        std::memcpy(out, img.host, elems * 2);
        std::free(img.host);
        return true;
    }, map);
}

// Host: the map applied to `weights` with the kernel's arithmetic must give the packer's own image of them.
bool repack_map_reproduces_packer(const marl_qnet_desc &desc, const float *weights, size_t n_params)
{
    std::vector<int32_t> map;
    PackedImage layout{};
    if (!build_repack_map(desc, n_params, &map, &layout)) return false;
    PackedImage img{};
    if (!pack_network(desc, weights, &img)) return false;
    const uint16_t *want = reinterpret_cast<const uint16_t *>(img.host);
    auto rne = [](float v) {
        uint32_t b;
        std::memcpy(&b, &v, 4);
        b += 0x7FFFu + ((b >> 16) & 1u);
        return (uint16_t)(b >> 16);
    };
    bool same = map.size() == img.off_w2_plain / 2;
    for (size_t e = 0; same && e < map.size(); ++e) {
        uint16_t got = 0;
        if (map[e] != kNoSource) {
            const float v = weights[map[e] & (kLowPlane - 1)];
            const uint16_t hi = rne(v);
            got = (map[e] & kLowPlane) ? rne(v - bf16_to_float(hi)) : hi;
        }
        same = got == want[e];
    }
    std::free(img.host);
    return same;
}

hipError_t launch_sgd_and_fragments(float *weights, const float *grad, float lr, size_t n_params, const int32_t *map_dev,
                                    size_t map_elems, void *image_dev, hipStream_t stream, const UpdateRule &rule)
{
    const dim3 grid((unsigned)((n_params + 255) / 256));
    if (rule.sq_avg) hipLaunchKernelGGL(rmsprop_kernel, grid, dim3(256), 0, stream, weights, grad, rule.sq_avg, lr, rule.alpha, rule.eps, n_params);
    else hipLaunchKernelGGL(sgd_kernel, grid, dim3(256), 0, stream, weights, grad, lr, n_params);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL(repack_frag_kernel, dim3((unsigned)((map_elems + 255) / 256)), dim3(256), 0, stream, weights, map_dev,
                       static_cast<uint16_t *>(image_dev), map_elems);
    return hipGetLastError();
}

hipError_t launch_copy_refresh(const float *weights, const int32_t *src_dev, size_t n, float *dst, hipStream_t stream)
{
    hipLaunchKernelGGL(copy_map_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, weights, src_dev, dst, n);
    return hipGetLastError();
}

hipError_t launch_sgd_step(const marl_qnet_desc &desc, const PackedImage &layout, int planes, const int32_t *map_dev,
                           size_t map_elems, void *image_dev, float *weights, const float *grad, size_t n_params, float lr,
                           hipStream_t stream, const UpdateRule &rule)
{
    const dim3 grid((unsigned)((n_params + 255) / 256));
    if (rule.sq_avg) hipLaunchKernelGGL(rmsprop_kernel, grid, dim3(256), 0, stream, weights, grad, rule.sq_avg, lr, rule.alpha, rule.eps, n_params);
    else hipLaunchKernelGGL(sgd_kernel, grid, dim3(256), 0, stream, weights, grad, lr, n_params);
    hipError_t err = hipGetLastError();
    if (err != hipSuccess) return err;
    TableArgs t{};
    t.w = weights; t.image = static_cast<char *>(image_dev);
    t.off_w2_plain = layout.off_w2_plain; t.off_bias1 = layout.off_bias1; t.off_b1_plain = layout.off_b1_plain; t.off_bias_r = layout.off_bias_r;
    t.off_bias_z = layout.off_bias_z; t.off_bias_in = layout.off_bias_in; t.off_bias_hn = layout.off_bias_hn;
    t.off_b2 = layout.off_b2;
    t.N = desc.n_agents; t.D = desc.obs_dim; t.A = desc.n_actions; t.H = desc.hidden; t.planes = planes;
    const int widest = std::max(std::max(t.A * t.H, t.N * t.H), std::max(t.H, t.A));
    const unsigned frag_blocks = (unsigned)((map_elems + 255) / 256), table_blocks = (unsigned)((widest + 255) / 256);
    hipLaunchKernelGGL(repack_image_kernel, dim3(frag_blocks + table_blocks), dim3(256), 0, stream, weights, map_dev,
                       static_cast<uint16_t *>(image_dev), map_elems, frag_blocks, t);
    return hipGetLastError();
}

}  // namespace marl
