// Chunk importance scores (Sec. 3.3 of the TokenSwift paper, Eq. 2), for gfx950:
//   scores[h][c] = scale * mean_{t in chunk c} sum_{j in group h} q_j . K[h][t].
// Eq. 2 is linear in both arguments, so the g query heads of the group are summed once
// (qbar), the keys of a chunk are summed as they stream in, and one dot product finishes the
// chunk.  The pass reads K exactly once and is bound by HBM bandwidth: one wavefront per
// chunk, lane = (row%4, 16-byte slice), so each load instruction fetches four whole 256-byte
// key rows, 16 of them in flight per lane.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

template <int G>
__global__ void __launch_bounds__(256) scores_kernel(const ScoresParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int c = lane & 15;      // 16-byte slice of a key row
    const int r = lane >> 4;      // row within a group of four
    const int64_t chunk = (int64_t)blockIdx.x * 4 + wave;
    const int h = blockIdx.y;
    if (chunk >= p.n_chunks) return;

    const int64_t t_begin = chunk * p.chunk_size;
    int64_t t_end = t_begin + p.chunk_size;
    if (t_end > p.n_tokens) t_end = p.n_tokens;

    float qbar[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int jj = 0; jj < G; ++jj) {
        const u32x4 raw = *reinterpret_cast<const u32x4 *>(p.q + ((int64_t)h * G + jj) * kHeadDim + c * 8);
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            qbar[2 * w] += bf16lo_to_f32(raw[w]);
            qbar[2 * w + 1] += bf16hi_to_f32(raw[w]);
        }
    }

    const uint16_t *kbase = p.k + (int64_t)h * p.stride_head + c * 8;
    float ksum[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int64_t t0 = t_begin; t0 < t_end; t0 += 64) {
        u32x4 raw[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const int64_t t = t0 + i * 4 + r;
            u32x4 z = {0u, 0u, 0u, 0u};
            raw[i] = (t < t_end) ? load_stream(kbase + t * p.stride_token) : z;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i)
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                ksum[2 * w] += bf16lo_to_f32(raw[i][w]);
                ksum[2 * w + 1] += bf16hi_to_f32(raw[i][w]);
            }
    }
    float d = 0.f;
#pragma unroll
    for (int x = 0; x < 8; ++x) d = fmaf(qbar[x], ksum[x], d);
    d = wave_sum(d);
    if (lane == 0) p.scores[(int64_t)h * p.n_chunks + chunk] = p.scale * d / (float)(t_end - t_begin);
}

template <int G>
hipError_t launch_g(const ScoresParams &p, hipStream_t stream)
{
    dim3 grid((unsigned)((p.n_chunks + 3) / 4), p.n_kv_heads);
    hipLaunchKernelGGL(scores_kernel<G>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_scores(const ScoresParams &p, hipStream_t stream)
{
    switch (p.group) {
        case 1: return launch_g<1>(p, stream);
        case 2: return launch_g<2>(p, stream);
        case 3: return launch_g<3>(p, stream);
        case 4: return launch_g<4>(p, stream);
        case 5: return launch_g<5>(p, stream);
        case 6: return launch_g<6>(p, stream);
        case 7: return launch_g<7>(p, stream);
        case 8: return launch_g<8>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ts
