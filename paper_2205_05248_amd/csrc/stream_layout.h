// Order in which the decision-step and input-projection kernels consume weight fragments.
// Both kernels pull the weights through LDS in chunks of kChunkPlanes fragment planes (1 KiB
// each: 64 lanes x 8 bf16; a fragment has P planes), so the host lays the fragments out in
// exactly the order of use and pads every section to whole chunks.  The same formulas are used
// by the host packer (runtime H, P) and by the kernels (compile-time H, P).
//
//   fc1 section     chunks of KPC k-steps; inside a chunk [k-step][feature block][plane]
//   GRU section     per hidden block, chunks of k-steps; inside a chunk [k-step][matrix][plane]
//                   with matrix = W_ir, W_iz, W_in (+ W_hr, W_hz, W_hn for the decision step)
//   fc2 section     (decision step only) chunks of k-steps; inside a chunk [k-step][action block][plane]
#pragma once

namespace marl {

constexpr int kChunkPlanes = 24;
constexpr int kChunkVecs = kChunkPlanes * 64;   // 16-byte vectors per chunk

struct StreamDims {
    int kpc;   // fc1 k-steps per chunk
    int kpg;   // GRU k-steps per chunk, decision step (6 matrices)
    int cpf;   // GRU chunks per hidden block, decision step
    int kpj;   // GRU k-steps per chunk, input projection (3 matrices)
    int cpj;   // GRU chunks per hidden block, input projection
    int kpf;   // fc2 k-steps per chunk
    int ncf;   // fc2 chunks
};

constexpr int stream_min(int a, int b) { return a < b ? a : b; }

constexpr StreamDims stream_dims(int H, int P, int MB2)
{
    const int MB = H / 32, KCH = H / 16;
    StreamDims d{};
    d.kpc = kChunkPlanes / (MB * P);
    d.kpg = stream_min(kChunkPlanes / (6 * P), KCH);
    d.cpf = KCH / d.kpg;
    d.kpj = stream_min(kChunkPlanes / (3 * P), KCH);
    d.cpj = KCH / d.kpj;
    d.kpf = stream_min(kChunkPlanes / (MB2 * P), KCH);
    d.ncf = (KCH + d.kpf - 1) / d.kpf;
    return d;
}

}  // namespace marl
