// Host side: turn the packed fp32 weight vector of include/marl_qnet.h into the
// device image used by the kernels (MFMA operand fragments + fp32 bias tables).
#include <cstdlib>
#include <cstring>

#include "qnet_internal.h"

namespace marl {
namespace {

// fp32 -> bits of the nearest bf16 (ties to even).
uint16_t bf16_bits(float v)
{
    uint32_t b;
    std::memcpy(&b, &v, 4);
    if ((b & 0x7F800000u) == 0x7F800000u) {
        if (b & 0x007FFFFFu) b |= 0x00400000u;
        return (uint16_t)(b >> 16);
    }
    b += 0x7FFFu + ((b >> 16) & 1u);
    return (uint16_t)(b >> 16);
}

float bf16_value(uint16_t bits)
{
    uint32_t b = (uint32_t)bits << 16;
    float v;
    std::memcpy(&v, &b, 4);
    return v;
}

size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }

int perm_c(int p)   // position inside the K axis -> source feature, for inputs that are MFMA results
{
    const int kc = p / 16, g = (p / 8) % 2, idx = p % 8;
    return 16 * kc + 8 * (idx / 4) + 4 * g + idx % 4;
}

// W: M x K row-major with leading dimension ld.  Output: [ceil(M/32)][ceil(K/16)][planes][64][8] bf16.
void pack_frags(uint16_t *out, const float *W, int M, int K, int ld, bool use_perm_c, int planes)
{
    const int MB = (M + 31) / 32, KC = (K + 15) / 16;
    for (int mb = 0; mb < MB; ++mb)
        for (int kc = 0; kc < KC; ++kc)
            for (int lane = 0; lane < 64; ++lane)
                for (int idx = 0; idx < 8; ++idx) {
                    const int m = 32 * mb + lane % 32;
                    const int p = 16 * kc + 8 * (lane / 32) + idx;
                    const int k = use_perm_c ? perm_c(p) : p;
                    const float w = (m < M && k < K) ? W[(size_t)m * ld + k] : 0.0f;
                    const uint16_t hi = bf16_bits(w);
                    uint16_t *frag = out + ((size_t)(mb * KC + kc) * planes) * 512;
                    frag[lane * 8 + idx] = hi;
                    if (planes == 2) frag[512 + lane * 8 + idx] = bf16_bits(w - bf16_value(hi));
                }
}

}  // namespace

bool pack_network(const marl_qnet_desc &d, const float *w, PackedImage *out)
{
    const int N = d.n_agents, D = d.obs_dim, A = d.n_actions, H = d.hidden, Din = D + N;
    const int planes = d.weight_dtype == MARL_DTYPE_BF16 ? 1 : 2;
    const int kc1 = (D + 15) / 16, mb2 = (A + 31) / 32, FB = H / 32, KCH = H / 16;
    const float *W1 = w, *b1 = W1 + (size_t)H * Din, *Wih = b1 + H, *Whh = Wih + (size_t)3 * H * H;
    const float *bih = Whh + (size_t)3 * H * H, *bhh = bih + 3 * H, *W2 = bhh + 3 * H, *b2 = W2 + (size_t)A * H;

    const size_t frag_bytes = (size_t)planes * 1024;
    size_t off = 0;
    out->off_w1 = off;      off = align256(off + (size_t)FB * kc1 * frag_bytes);
    out->off_wih = off;     off = align256(off + (size_t)3 * FB * KCH * frag_bytes);
    out->off_whh = off;     off = align256(off + (size_t)3 * FB * KCH * frag_bytes);
    out->off_w2 = off;      off = align256(off + (size_t)mb2 * KCH * frag_bytes);
    out->off_bias1 = off;   off = align256(off + sizeof(float) * (size_t)N * H);
    out->off_bias_r = off;  off = align256(off + sizeof(float) * H);
    out->off_bias_z = off;  off = align256(off + sizeof(float) * H);
    out->off_bias_in = off; off = align256(off + sizeof(float) * H);
    out->off_bias_hn = off; off = align256(off + sizeof(float) * H);
    out->off_b2 = off;      off = align256(off + sizeof(float) * 32 * mb2);
    out->bytes = off;
    out->kc1 = kc1; out->mb2 = mb2; out->planes = planes;
    char *img = static_cast<char *>(std::calloc(off, 1));
    if (!img) return false;
    out->host = img;

    pack_frags(reinterpret_cast<uint16_t *>(img + out->off_w1), W1, H, D, Din, false, planes);
    for (int gate = 0; gate < 3; ++gate) {
        const size_t per_gate = (size_t)FB * KCH * frag_bytes;
        pack_frags(reinterpret_cast<uint16_t *>(img + out->off_wih + gate * per_gate), Wih + (size_t)gate * H * H, H, H, H, true, planes);
        pack_frags(reinterpret_cast<uint16_t *>(img + out->off_whh + gate * per_gate), Whh + (size_t)gate * H * H, H, H, H, true, planes);
    }
    pack_frags(reinterpret_cast<uint16_t *>(img + out->off_w2), W2, A, H, H, true, planes);

    // The agent-id column of W1 is a per-agent bias.  A bf16 network uses the rounded weight.
    float *bias1 = reinterpret_cast<float *>(img + out->off_bias1);
    for (int n = 0; n < N; ++n)
        for (int j = 0; j < H; ++j) {
            float col = W1[(size_t)j * Din + D + n];
            if (planes == 1) col = bf16_value(bf16_bits(col));
            bias1[(size_t)n * H + j] = b1[j] + col;
        }
    float *br = reinterpret_cast<float *>(img + out->off_bias_r), *bz = reinterpret_cast<float *>(img + out->off_bias_z);
    float *bin = reinterpret_cast<float *>(img + out->off_bias_in), *bhn = reinterpret_cast<float *>(img + out->off_bias_hn);
    for (int j = 0; j < H; ++j) {
        br[j] = bih[j] + bhh[j];
        bz[j] = bih[H + j] + bhh[H + j];
        bin[j] = bih[2 * H + j];
        bhn[j] = bhh[2 * H + j];
    }
    std::memcpy(img + out->off_b2, b2, sizeof(float) * A);
    return true;
}

}  // namespace marl
