// Attention of one query token per head over the selected chunks of the KV cache (the
// partial cache C_p of Alg. 1, used by the drafting forward pass), as flash-decoding split
// along the keys, for gfx950.
//
// Only g <= 8 query rows share a KV head here, so this is not a matrix contraction: plain
// VALU.  A 16-lane row of a wavefront owns one segment of 8 consecutive tokens of one selected
// chunk; lane c of the row holds the 16-byte slice c of each key/value row, so one wavefront
// load instruction fetches four complete 256-byte rows.  All keys and values of the segment
// are requested up front (16 loads in flight per lane).  The g rows of the group share them:
// a key or value row is unpacked once and used by all g rows; logits are reduced across the
// 16-lane row with DPP; the whole segment is resident, so its softmax needs no running rescale.  The 16 segments
// of a workgroup are merged through LDS in one step; the workgroup writes one (m, l,
// unnormalised O) per query head of the group and combine_kernel merges the workgroups.
// The chunks are read in place through chunk_idx: no gather copy.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

constexpr int kSegKeys = 8;
constexpr int kSegsPerWg = 16;

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
    extern __shared__ __attribute__((aligned(16))) float smem[];
    float *o_lds = smem;                                   // [16 segments][G][128]
    float *ml_lds = smem + kSegsPerWg * G * kHeadDim;      // [16 segments][G][2]
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int c = lane & 15;                               // 16-byte slice of a row
    const int seg_in_block = tid >> 4;                     // 16 segments per workgroup
    const int segment = blockIdx.x * kSegsPerWg + seg_in_block;    // segment id within the head
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
        kraw[kk] = (t < t_end) ? load_stream(kbase + t * p.stride_token) : z;
    }
#pragma unroll
    for (int kk = 0; kk < kSegKeys; ++kk) {
        const int64_t t = t_begin + kk;
        u32x4 z = {0u, 0u, 0u, 0u};
        vraw[kk] = (t < t_end) ? load_stream(vbase + t * p.stride_token) : z;
    }
    float qf[G][8];
#pragma unroll
    for (int jj = 0; jj < G; ++jj) unpack8(*reinterpret_cast<const u32x4 *>(p.q + ((int64_t)h * G + jj) * kHeadDim + c * 8), qf[jj]);

    // logits of the g rows against the 8 keys: this lane's 8 dimensions (a key row is unpacked once
    // for all g rows), then the sum over the row.  (v_dot2c_f32_bf16 on the packed operands would
    // save the unpacking, but its products are not carried in full precision: the logits came
    // out ~1e-2 off.)
    float w[G][kSegKeys];
#pragma unroll
    for (int kk = 0; kk < kSegKeys; ++kk) {
        float kf[8];
        unpack8(kraw[kk], kf);
#pragma unroll
        for (int jj = 0; jj < G; ++jj) {
            float d = 0.f;
#pragma unroll
            for (int x = 0; x < 8; ++x) d = fmaf(qf[jj][x], kf[x], d);
            w[jj][kk] = d;
        }
    }
    float m[G], l[G];
#pragma unroll
    for (int jj = 0; jj < G; ++jj) {
        m[jj] = kNegBig;
#pragma unroll
        for (int kk = 0; kk < kSegKeys; ++kk) {
            const float d = row16_sum(w[jj][kk]) * p.scale_log2;
            w[jj][kk] = (t_begin + kk < t_end) ? d : -INFINITY;
            m[jj] = fmaxf(m[jj], w[jj][kk]);
        }
        l[jj] = 0.f;
#pragma unroll
        for (int kk = 0; kk < kSegKeys; ++kk) {
            w[jj][kk] = fast_exp2(w[jj][kk] - m[jj]);   // 0 for masked keys, also when the row is idle
            l[jj] += w[jj][kk];
        }
    }
    float o[G][8];
#pragma unroll
    for (int jj = 0; jj < G; ++jj)
#pragma unroll
        for (int x = 0; x < 8; ++x) o[jj][x] = 0.f;
#pragma unroll
    for (int kk = 0; kk < kSegKeys; ++kk) {
        float vf[8];
        unpack8(vraw[kk], vf);
#pragma unroll
        for (int jj = 0; jj < G; ++jj)
#pragma unroll
            for (int x = 0; x < 8; ++x) o[jj][x] = fmaf(w[jj][kk], vf[x], o[jj][x]);
    }

    // merge the 16 segments of the workgroup (fixed order: deterministic)
#pragma unroll
    for (int jj = 0; jj < G; ++jj) {
        float *dst = o_lds + (seg_in_block * G + jj) * kHeadDim + c * 8;
        *reinterpret_cast<f32x4 *>(dst) = f32x4{o[jj][0], o[jj][1], o[jj][2], o[jj][3]};
        *reinterpret_cast<f32x4 *>(dst + 4) = f32x4{o[jj][4], o[jj][5], o[jj][6], o[jj][7]};
        if (c == 0) *reinterpret_cast<f32x2 *>(ml_lds + (seg_in_block * G + jj) * 2) = f32x2{m[jj], l[jj]};
    }
    __syncthreads();
    const int64_t prow = ((int64_t)h * p.n_part + blockIdx.x) * G;
    for (int idx = tid; idx < G * kHeadDim; idx += 256) {
        const int jj = idx >> 7, dim = idx & (kHeadDim - 1);
        float mstar = kNegBig;
#pragma unroll
        for (int s = 0; s < kSegsPerWg; ++s) mstar = fmaxf(mstar, ml_lds[(s * G + jj) * 2]);
        float acc = 0.f, lstar = 0.f;
#pragma unroll
        for (int s = 0; s < kSegsPerWg; ++s) {
            const float ws = fast_exp2(ml_lds[(s * G + jj) * 2] - mstar);
            lstar = fmaf(ws, ml_lds[(s * G + jj) * 2 + 1], lstar);
            acc = fmaf(ws, o_lds[(s * G + jj) * kHeadDim + dim], acc);
        }
        p.ws_o[(prow + jj) * kHeadDim + dim] = acc;
        if (dim == 0) *reinterpret_cast<f32x2 *>(p.ws_ml + (prow + jj) * 2) = f32x2{mstar, lstar};
    }
}

template <int G>
hipError_t launch_g(const PartialParams &p, hipStream_t stream)
{
    constexpr int lds_bytes = kSegsPerWg * G * (kHeadDim + 2) * (int)sizeof(float);
    static std::atomic<uint64_t> lds_allowed{0};
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(partial_kernel<G>), lds_bytes, lds_allowed);
        if (e != hipSuccess) return e;
    }
    dim3 grid(p.n_part, p.n_kv_heads);
    hipLaunchKernelGGL(partial_kernel<G>, grid, dim3(256), lds_bytes, stream, p);
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
