// Host side: turn the packed fp32 weight vector of include/marl_qnet.h into the
// device image used by the kernels (MFMA operand fragments + fp32 bias tables).
#include <cstdlib>
#include <cstring>

#include <vector>

#include "qnet_internal.h"
#include "stream_layout.h"

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

// 16x16x32 MFMA operand fragments (fused unroll): W is cut into fragments of 16 rows x 32 k.
// Fragment (mb, ks), lane l (q = l / 16, m = l % 16), idx = 0..7 holds W[16 mb + m][perm(32 ks + 8 q + idx)].
// perm is the identity for the first layer; for layers fed by an MFMA result it is
//   perm16(32 ks + 8 q + idx) = 32 ks + 16 (idx / 4) + 4 q + idx % 4,
// where the 16x16 accumulators of two adjacent feature blocks leave their values.
int perm16(int p)
{
    const int ks = p / 32, q = (p / 8) % 4, idx = p % 8;
    return 32 * ks + 16 * (idx / 4) + 4 * q + idx % 4;
}

}  // namespace

// Output: [ceil(M/16)][ceil(K/32)][planes][64][8] bf16.
void pack_frags16(uint16_t *out, const float *W, int M, int K, int ld, bool use_perm, int planes)
{
    const int MB = (M + 15) / 16, KS = (K + 31) / 32;
    for (int mb = 0; mb < MB; ++mb)
        for (int ks = 0; ks < KS; ++ks)
            for (int lane = 0; lane < 64; ++lane)
                for (int idx = 0; idx < 8; ++idx) {
                    const int m = 16 * mb + lane % 16;
                    const int p = 32 * ks + 8 * (lane / 16) + idx;
                    const int k = use_perm ? perm16(p) : p;
                    const float w = (m < M && k < K) ? W[(size_t)m * ld + k] : 0.0f;
                    const uint16_t hi = bf16_bits(w);
                    uint16_t *frag = out + ((size_t)(mb * KS + ks) * planes) * 512;
                    frag[lane * 8 + idx] = hi;
                    if (planes == 2) frag[512 + lane * 8 + idx] = bf16_bits(w - bf16_value(hi));
                }
}


bool pack_network(const marl_qnet_desc &d, const float *w, PackedImage *out)
{
    const int N = d.n_agents, D = d.obs_dim, A = d.n_actions, H = d.hidden, Din = D + N;
    const int planes = d.weight_dtype == MARL_DTYPE_BF16 ? 1 : 2;
    const int kc1 = (D + 15) / 16, mb2 = (A + 31) / 32, FB = H / 32, KCH = H / 16;
    const float *W1 = w, *b1 = W1 + (size_t)H * Din, *Wih = b1 + H, *Whh = Wih + (size_t)3 * H * H;
    const float *bih = Whh + (size_t)3 * H * H, *bhh = bih + 3 * H, *W2 = bhh + 3 * H, *b2 = W2 + (size_t)A * H;

    const size_t frag_bytes = (size_t)planes * 1024;
    const StreamDims sd = stream_dims(H, planes, mb2);
    const int nc1 = (kc1 + sd.kpc - 1) / sd.kpc;
    const int act_chunks = nc1 + FB * sd.cpf + sd.ncf, proj_chunks = nc1 + FB * sd.cpj;
    const size_t chunk_bytes = (size_t)kChunkPlanes * 1024;
    size_t off = 0;
    out->off_act = off;     off = align256(off + (size_t)act_chunks * chunk_bytes);
    out->off_proj = off;    off = align256(off + (size_t)proj_chunks * chunk_bytes);
    out->off_whh = off;     off = align256(off + (size_t)3 * FB * KCH * frag_bytes);
    out->off_w2 = off;      off = align256(off + (size_t)mb2 * KCH * frag_bytes);
    const int ks1 = (D + 31) / 32, ab = (A + 15) / 16, FBK = H / 16, KS = H / 32;
    out->off_w1_16 = off;   off = align256(off + (size_t)FBK * ks1 * frag_bytes);
    out->off_wih_16 = off;  off = align256(off + (size_t)3 * FBK * KS * frag_bytes);
    out->off_whh_16 = off;  off = align256(off + (size_t)3 * FBK * KS * frag_bytes);
    out->off_w2_16 = off;   off = align256(off + (size_t)ab * KS * frag_bytes);
    const int ks1x = (Din + 31) / 32;
    out->off_w1x_16 = off;  off = align256(off + (size_t)FBK * ks1x * frag_bytes);
    out->off_wihT_16 = off; off = align256(off + (size_t)FBK * 3 * KS * frag_bytes);
    out->off_whhT_16 = off; off = align256(off + (size_t)FBK * 3 * KS * frag_bytes);
    out->off_w2_plain = off; off = align256(off + sizeof(float) * (size_t)A * H);
    out->off_bias1 = off;   off = align256(off + sizeof(float) * (size_t)N * H);
    out->off_b1_plain = off; off = align256(off + sizeof(float) * H);
    out->off_bias_r = off;  off = align256(off + sizeof(float) * H);
    out->off_bias_z = off;  off = align256(off + sizeof(float) * H);
    out->off_bias_in = off; off = align256(off + sizeof(float) * H);
    out->off_bias_hn = off; off = align256(off + sizeof(float) * H);
    out->off_b2 = off;      off = align256(off + sizeof(float) * 32 * mb2);
    out->bytes = off;
    out->kc1 = kc1; out->mb2 = mb2; out->planes = planes;
    out->nc1 = nc1; out->act_chunks = act_chunks; out->proj_chunks = proj_chunks;
    char *img = static_cast<char *>(std::calloc(off, 1));
    if (!img) return false;
    out->host = img;

    // Fragment arrays per matrix: [block][k-step][plane][512 bf16].
    const size_t frag_elems = (size_t)planes * 512;
    std::vector<uint16_t> w1f((size_t)FB * kc1 * frag_elems), wihf((size_t)3 * FB * KCH * frag_elems);
    uint16_t *whhf = reinterpret_cast<uint16_t *>(img + out->off_whh);
    uint16_t *w2f = reinterpret_cast<uint16_t *>(img + out->off_w2);
    pack_frags(w1f.data(), W1, H, D, Din, false, planes);
    for (int gate = 0; gate < 3; ++gate) {
        const size_t per_gate = (size_t)FB * KCH * frag_elems;
        pack_frags(wihf.data() + gate * per_gate, Wih + (size_t)gate * H * H, H, H, H, true, planes);
        pack_frags(whhf + gate * per_gate, Whh + (size_t)gate * H * H, H, H, H, true, planes);
    }
    pack_frags(w2f, W2, A, H, H, true, planes);

    // Streams: copy fragments into their order of use; k-steps beyond a matrix stay zero.
    auto frag_w1 = [&](int mb, int kc) { return kc < kc1 ? w1f.data() + ((size_t)mb * kc1 + kc) * frag_elems : nullptr; };
    auto frag_gru = [&](const uint16_t *base, int gate, int fb, int kc) { return base + ((size_t)(gate * FB + fb) * KCH + kc) * frag_elems; };
    auto frag_w2 = [&](int mb, int kc) { return w2f + ((size_t)mb * KCH + kc) * frag_elems; };
    for (int which = 0; which < 2; ++which) {           // 0: decision step, 1: input projection
        uint16_t *dst = reinterpret_cast<uint16_t *>(img + (which ? out->off_proj : out->off_act));
        const size_t chunk_elems = (size_t)kChunkPlanes * 512;
        int chunk = 0;
        auto put = [&](int slot, const uint16_t *frag) {   // slot = fragment index inside the chunk
            if (frag) std::memcpy(dst + chunk * chunk_elems + (size_t)slot * frag_elems, frag, frag_elems * 2);
        };
        for (int c = 0; c < nc1; ++c, ++chunk)
            for (int kk = 0; kk < sd.kpc; ++kk)
                for (int mb = 0; mb < FB; ++mb) put(kk * FB + mb, frag_w1(mb, c * sd.kpc + kk));
        const int nmat = which ? 3 : 6, kper = which ? sd.kpj : sd.kpg, cper = which ? sd.cpj : sd.cpf;
        for (int fb = 0; fb < FB; ++fb)
            for (int cc = 0; cc < cper; ++cc, ++chunk)
                for (int kk = 0; kk < kper; ++kk)
                    for (int m = 0; m < nmat; ++m) {
                        const int kc = cc * kper + kk;
                        put(kk * nmat + m, m < 3 ? frag_gru(wihf.data(), m, fb, kc) : frag_gru(whhf, m - 3, fb, kc));
                    }
        if (!which)
            for (int cf = 0; cf < sd.ncf; ++cf, ++chunk)
                for (int kk = 0; kk < sd.kpf; ++kk)
                    for (int mb = 0; mb < mb2; ++mb) {
                        const int kc = cf * sd.kpf + kk;
                        if (kc < KCH) put(kk * mb2 + mb, frag_w2(mb, kc));
                    }
    }

    // Fused unroll: 16-row tiles, 16x16x32 fragments.
    {
        pack_frags16(reinterpret_cast<uint16_t *>(img + out->off_w1_16), W1, H, D, Din, false, planes);
        const size_t per_gate16 = (size_t)FBK * KS * frag_elems;
        for (int gate = 0; gate < 3; ++gate) {
            pack_frags16(reinterpret_cast<uint16_t *>(img + out->off_wih_16) + gate * per_gate16,
                         Wih + (size_t)gate * H * H, H, H, H, true, planes);
            pack_frags16(reinterpret_cast<uint16_t *>(img + out->off_whh_16) + gate * per_gate16,
                         Whh + (size_t)gate * H * H, H, H, H, true, planes);
        }
        pack_frags16(reinterpret_cast<uint16_t *>(img + out->off_w2_16), W2, A, H, H, true, planes);
        // the same first layer with the agent-id columns kept in the product (streaming decision step)
        pack_frags16(reinterpret_cast<uint16_t *>(img + out->off_w1x_16), W1, H, Din, Din, false, planes);
    }

    // Backward pass: W_ih^T and W_hh^T as [H, 3H] matrices (row k, column gate H + j), and fc2 as it is.
    {
        std::vector<float> wt((size_t)H * 3 * H);
        for (int which = 0; which < 2; ++which) {
            const float *W = which ? Whh : Wih;
            for (int g = 0; g < 3 * H; ++g)
                for (int k = 0; k < H; ++k) wt[(size_t)k * 3 * H + g] = W[(size_t)g * H + k];
            pack_frags16(reinterpret_cast<uint16_t *>(img + (which ? out->off_whhT_16 : out->off_wihT_16)), wt.data(), H,
                         3 * H, 3 * H, true, planes);
        }
        float *w2p = reinterpret_cast<float *>(img + out->off_w2_plain);
        for (size_t i = 0; i < (size_t)A * H; ++i) w2p[i] = planes == 1 ? bf16_value(bf16_bits(W2[i])) : W2[i];
    }

    // The agent-id column of W1 is a per-agent bias.  A bf16 network uses the rounded weight.
    float *bias1 = reinterpret_cast<float *>(img + out->off_bias1);
    for (int n = 0; n < N; ++n)
        for (int j = 0; j < H; ++j) {
            float col = W1[(size_t)j * Din + D + n];
            if (planes == 1) col = bf16_value(bf16_bits(col));
            bias1[(size_t)n * H + j] = b1[j] + col;
        }
    std::memcpy(img + out->off_b1_plain, b1, sizeof(float) * H);
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
