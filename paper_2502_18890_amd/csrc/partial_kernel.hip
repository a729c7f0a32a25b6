// Attention of one query token per head over the selected chunks of the KV cache (the
// partial cache C_p of Alg. 1, used by the drafting forward pass), as flash-decoding split
// along the keys, for gfx950.
//
// Only g <= 8 query rows share a KV head here, so this is not a matrix contraction: plain
// fp32 VALU.  A 16-lane row of a wavefront owns one segment of 16 consecutive tokens of one
// selected chunk; lane c of the row holds the 16-byte slice c of each key/value row, so one
// wavefront load instruction fetches four complete 256-byte rows.  All 16 keys and values of
// the segment are requested up front (32 loads in flight per lane).  Dot products are reduced
// across the row with DPP; since the whole segment is resident, its softmax needs no running
// rescale.  Every segment writes (m, l, unnormalised O) per query head of the group and
// combine_kernel merges them.  The chunks are read in place through chunk_idx: no gather copy.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

constexpr int kSegKeys = 16;

__device__ __forceinline__ void unpack8(const u32x4 &raw, float (&f)[8])
{
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        f[2 * w] = bf16lo_to_f32(raw[w]);
        f[2 * w + 1] = bf16hi_to_f32(raw[w]);
    }
}

template <int G>
__global__ void __launch_bounds__(256) partial_kernel(const PartialParams p)
{
    const int lane = threadIdx.x & 63;
    const int c = lane & 15;                               // 16-byte slice of a row
    const int seg_in_block = threadIdx.x >> 4;             // 16 segments per workgroup
    const int part = blockIdx.x * 16 + seg_in_block;       // segment id within the head
    const int h = blockIdx.y;
    if (part >= p.n_part) return;                          // whole 16-lane rows leave together

    const int sel = part / p.segs_per_chunk;
    const int seg = part - sel * p.segs_per_chunk;
    const int64_t chunk = p.chunk_idx[(int64_t)h * p.n_sel + sel];
    const int64_t t_begin = chunk * p.chunk_size + (int64_t)seg * kSegKeys;
    int64_t t_end = (chunk + 1) * p.chunk_size;
    if (t_end > p.n_tokens) t_end = p.n_tokens;
    if (t_begin + kSegKeys < t_end) t_end = t_begin + kSegKeys;

    const uint16_t *kbase = p.k + (int64_t)h * p.stride_head + c * 8;
    const uint16_t *vbase = p.v + (int64_t)h * p.stride_head + c * 8;

    u32x4 kraw[kSegKeys], vraw[kSegKeys];
#pragma unroll
    for (int kk = 0; kk < kSegKeys; ++kk) {
        const int64_t t = t_begin + kk;
        u32x4 z = {0u, 0u, 0u, 0u};
        kraw[kk] = (t < t_end) ? *reinterpret_cast<const u32x4 *>(kbase + t * p.stride_token) : z;
    }
#pragma unroll
    for (int kk = 0; kk < kSegKeys; ++kk) {
        const int64_t t = t_begin + kk;
        u32x4 z = {0u, 0u, 0u, 0u};
        vraw[kk] = (t < t_end) ? *reinterpret_cast<const u32x4 *>(vbase + t * p.stride_token) : z;
    }

    const int64_t prow = ((int64_t)h * p.n_part + part) * G;
#pragma unroll 1
    for (int jj = 0; jj < G; ++jj) {
        float qf[8];
        unpack8(*reinterpret_cast<const u32x4 *>(p.q + ((int64_t)h * G + jj) * kHeadDim + c * 8), qf);
        float t[kSegKeys];
        float m = kNegBig;
#pragma unroll
        for (int kk = 0; kk < kSegKeys; ++kk) {
            float kf[8];
            unpack8(kraw[kk], kf);
            float d = 0.f;
#pragma unroll
            for (int x = 0; x < 8; ++x) d = fmaf(qf[x], kf[x], d);
            d = row16_sum(d) * p.scale_log2;
            t[kk] = (t_begin + kk < t_end) ? d : -INFINITY;
            m = fmaxf(m, t[kk]);
        }
        float l = 0.f;
        float o[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < kSegKeys; ++kk) {
            const float pk = fast_exp2(t[kk] - m);
            l += pk;
            float vf[8];
            unpack8(vraw[kk], vf);
#pragma unroll
            for (int x = 0; x < 8; ++x) o[x] = fmaf(pk, vf[x], o[x]);
        }
        float *orow = p.ws_o + (prow + jj) * kHeadDim + c * 8;
        *reinterpret_cast<f32x4 *>(orow) = f32x4{o[0], o[1], o[2], o[3]};
        *reinterpret_cast<f32x4 *>(orow + 4) = f32x4{o[4], o[5], o[6], o[7]};
        if (c == 0) *reinterpret_cast<f32x2 *>(p.ws_ml + (prow + jj) * 2) = f32x2{m, l};
    }
}

template <int G>
hipError_t launch_g(const PartialParams &p, hipStream_t stream)
{
    dim3 grid((p.n_part + 15) / 16, p.n_kv_heads);
    hipLaunchKernelGGL(partial_kernel<G>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_partial(const PartialParams &p, hipStream_t stream)
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
