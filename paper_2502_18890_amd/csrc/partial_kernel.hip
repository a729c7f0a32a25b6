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
// rescale.  The 16 segments of a workgroup are merged through LDS; the workgroup writes one
// (m, l, unnormalised O) per query head of the group and combine_kernel merges the workgroups.
// The chunks are read in place through chunk_idx: no gather copy.
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
    __shared__ float o_lds[16][kHeadDim];
    __shared__ float ml_lds[16][2];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int c = lane & 15;                               // 16-byte slice of a row
    const int seg_in_block = tid >> 4;                     // 16 segments per workgroup
    const int segment = blockIdx.x * 16 + seg_in_block;    // segment id within the head
    const int h = blockIdx.y;
    const bool valid = segment < p.n_seg;

    int64_t t_begin = 0, t_end = 0;                        // empty range for an idle row
    if (valid) {
        const int sel = segment / p.segs_per_chunk;
        const int seg = segment - sel * p.segs_per_chunk;
        const int64_t chunk = p.chunk_idx[(int64_t)h * p.n_sel + sel];
        t_begin = chunk * p.chunk_size + (int64_t)seg * kSegKeys;
        t_end = (chunk + 1) * p.chunk_size;
        if (t_end > p.n_tokens) t_end = p.n_tokens;
        if (t_begin + kSegKeys < t_end) t_end = t_begin + kSegKeys;
    }

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

    const int64_t prow = ((int64_t)h * p.n_part + blockIdx.x) * G;
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
            const float pk = fast_exp2(t[kk] - m);   // 0 for masked keys, also when the row is idle
            l += pk;
            float vf[8];
            unpack8(vraw[kk], vf);
#pragma unroll
            for (int x = 0; x < 8; ++x) o[x] = fmaf(pk, vf[x], o[x]);
        }
        // merge the 16 segments of the workgroup (fixed order: deterministic)
        *reinterpret_cast<f32x4 *>(&o_lds[seg_in_block][c * 8]) = f32x4{o[0], o[1], o[2], o[3]};
        *reinterpret_cast<f32x4 *>(&o_lds[seg_in_block][c * 8 + 4]) = f32x4{o[4], o[5], o[6], o[7]};
        if (c == 0) {
            ml_lds[seg_in_block][0] = m;
            ml_lds[seg_in_block][1] = l;
        }
        __syncthreads();
        if (tid < kHeadDim) {
            float mstar = kNegBig;
#pragma unroll
            for (int s = 0; s < 16; ++s) mstar = fmaxf(mstar, ml_lds[s][0]);
            float acc = 0.f, lstar = 0.f;
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const float w = fast_exp2(ml_lds[s][0] - mstar);
                lstar = fmaf(w, ml_lds[s][1], lstar);
                acc = fmaf(w, o_lds[s][tid], acc);
            }
            p.ws_o[(prow + jj) * kHeadDim + tid] = acc;
            if (tid == 0) *reinterpret_cast<f32x2 *>(p.ws_ml + (prow + jj) * 2) = f32x2{mstar, lstar};
        }
        __syncthreads();
    }
}

template <int G>
hipError_t launch_g(const PartialParams &p, hipStream_t stream)
{
    dim3 grid(p.n_part, p.n_kv_heads);
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
