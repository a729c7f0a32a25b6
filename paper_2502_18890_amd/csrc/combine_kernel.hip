// Merge of split-K attention partials: for each query row, partial i carries the maximum
// logit m_i (exp2 domain), l_i = sum exp2(logit - m_i) and O_i = sum exp2(logit - m_i) * v over
// its own keys.  Softmax attention over the union of the key sets is
//   m* = max m_i,  l* = sum l_i 2^(m_i - m*),  out = sum O_i 2^(m_i - m*) / l*,
// and the natural-log sum of exponentials is (m* + log2 l*) ln 2.
// One wavefront per row, two output columns per lane; the weights are computed once, one partial
// per lane, and broadcast as the partials stream in, sixteen loads in flight.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

__global__ void __launch_bounds__(256) combine_kernel(const CombineParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int h = blockIdx.y;
    const int row_blocks = (p.n_rows + 3) / 4;
    if ((int)blockIdx.x >= row_blocks) {
        // Workgroups behind the row blocks: chunk scores (Eq. 2 with the first tree node's queries) from the
        // per-tile sums of raw logits that the split kernel left: one chunk per thread.
        const int64_t c = (int64_t)(blockIdx.x - row_blocks) * 256 + threadIdx.x;
        if (c >= p.n_chunks) return;
        const int tiles_per_chunk = p.chunk_size / 32;
        const int64_t n_tiles = (p.n_tokens + 31) / 32;
        const float *ts = p.tile_sums + (int64_t)h * p.tile_sums_stride;
        float s = 0.f;
        for (int i = 0; i < tiles_per_chunk; ++i) {
            const int64_t t = c * tiles_per_chunk + i;
            if (t < n_tiles) s += ts[t];
        }
        int64_t count = p.n_tokens - c * p.chunk_size;
        if (count > p.chunk_size) count = p.chunk_size;
        p.scores[(int64_t)h * p.n_chunks + c] = p.scale * s / (float)count;
        return;
    }
    const int row = blockIdx.x * 4 + wave;
    if (row >= p.n_rows) return;   // whole wavefront leaves together

    const int64_t pitch = p.row_pitch;
    const int64_t first = (int64_t)h * p.n_part * pitch + row;   // partial pp at first + pp*pitch

    // Lane pp holds the weight of partials pp, pp+64, ...: w = 2^(m_pp - m*), and l* = sum w l.
    f32x2 acc = {0.f, 0.f};
    float lsum = 0.f;
    float mstar = kNegBig;
    auto o_at = [&](int pp) {
        return *reinterpret_cast<const f32x2 *>(p.ws_o + (first + (int64_t)pp * pitch) * kHeadDim + lane * 2);
    };
    if (p.n_part <= 64) {
        // The usual case.  The first sixteen partials' outputs are requested before the (m, l) pairs are
        // needed, so the two rounds of memory latency overlap instead of following each other.
        f32x2 ml = {kNegBig, 0.f};
        if (lane < p.n_part) ml = *reinterpret_cast<const f32x2 *>(p.ws_ml + (first + (int64_t)lane * pitch) * 2);
        f32x2 o[16];
#pragma unroll
        for (int u = 0; u < 16; ++u) o[u] = u < p.n_part ? o_at(u) : f32x2{0.f, 0.f};
        mstar = wave_max(ml[0]);
        const float w = lane < p.n_part ? fast_exp2(ml[0] - mstar) : 0.f;
        lsum = w * ml[1];
#pragma unroll
        for (int u = 0; u < 16; ++u) acc += o[u] * __shfl(w, u, 64);   // weight 0 beyond n_part
        int u0 = 16;
        for (; u0 + 16 <= p.n_part; u0 += 16) {
#pragma unroll
            for (int u = 0; u < 16; ++u) o[u] = o_at(u0 + u);
#pragma unroll
            for (int u = 0; u < 16; ++u) acc += o[u] * __shfl(w, u0 + u, 64);
        }
        for (; u0 < p.n_part; ++u0) acc += o_at(u0) * __shfl(w, u0, 64);
    } else {
        for (int pp = lane; pp < p.n_part; pp += 64)
            mstar = fmaxf(mstar, p.ws_ml[(first + (int64_t)pp * pitch) * 2]);
        mstar = wave_max(mstar);
        for (int base = 0; base < p.n_part; base += 64) {
            float w = 0.f;
            if (base + lane < p.n_part) {
                const f32x2 ml = *reinterpret_cast<const f32x2 *>(p.ws_ml + (first + (int64_t)(base + lane) * pitch) * 2);
                w = fast_exp2(ml[0] - mstar);
                lsum = fmaf(w, ml[1], lsum);
            }
            const int n_here = p.n_part - base < 64 ? p.n_part - base : 64;
            int u0 = 0;
            for (; u0 + 16 <= n_here; u0 += 16) {   // sixteen partials in flight
                f32x2 o[16];
#pragma unroll
                for (int u = 0; u < 16; ++u) o[u] = o_at(base + u0 + u);
#pragma unroll
                for (int u = 0; u < 16; ++u) acc += o[u] * __shfl(w, u0 + u, 64);
            }
            for (; u0 < n_here; ++u0) acc += o_at(base + u0) * __shfl(w, u0, 64);
        }
    }
    const float lstar = wave_sum(lsum);
    const int node = row / p.group, jj = row % p.group;
    const int64_t orow = (int64_t)node * p.n_q_heads + h * p.group + jj;
    const float inv = 1.0f / lstar;
    f32x2 res = {acc[0] * inv, acc[1] * inv};
    *reinterpret_cast<f32x2 *>(p.out + orow * kHeadDim + lane * 2) = res;
    if (p.lse != nullptr && lane == 0) p.lse[orow] = (mstar + fast_log2(lstar)) * kLn2;
}

}  // namespace

hipError_t launch_combine(const CombineParams &p, hipStream_t stream)
{
    const unsigned score_blocks = p.tile_sums ? (unsigned)((p.n_chunks + 255) / 256) : 0u;
    dim3 grid((p.n_rows + 3) / 4 + score_blocks, p.n_kv_heads);
    hipLaunchKernelGGL(combine_kernel, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace ts
