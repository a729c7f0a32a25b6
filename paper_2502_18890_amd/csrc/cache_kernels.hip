// Cache maintenance around the attention passes of TokenSwift (Alg. 1: update of C_full with
// the accepted tokens, eviction inside C_p, rebuild of C_p; Sec. 3.3 "Dynamic KV Cache
// Updates"), for gfx950.  All of these move or reduce rows of 256 bytes; a 16-lane group
// handles one row with 128-bit accesses, so a wavefront instruction covers four whole rows.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

// ---- append the accepted path to the full cache -----------------------------------------------
// grid (n_accepted, n_kv_heads), 64 threads: lanes 0..15 copy the key row, 16..31 the value row.
__global__ void __launch_bounds__(64) append_kernel(const AppendParams p)
{
    const int i = blockIdx.x, h = blockIdx.y;
    const int lane = threadIdx.x;
    if (lane >= 32) return;
    const int c = lane & 15;
    const bool is_v = lane >= 16;
    const uint16_t *src = (is_v ? p.v_tree : p.k_tree) + ((int64_t)p.accepted[i] * p.n_kv_heads + h) * kHeadDim + c * 8;
    uint16_t *dst = (is_v ? p.v : p.k) + (int64_t)h * p.stride_head + (p.n_tokens + i) * p.stride_token + c * 8;
    *reinterpret_cast<u32x4 *>(dst) = *reinterpret_cast<const u32x4 *>(src);
}

// ---- admit new chunks at the tail of the chunk lists --------------------------------------------
// One workgroup per KV head.  New chunk c owns position n_sel - 1 - (c - base_chunk).  The chunks are
// taken one after the other (a swap may move an entry that a later chunk then evicts); for each, all
// threads look for c in the list and thread 0 applies the one change.
__global__ void __launch_bounds__(256) admit_kernel(int32_t *chunk_idx, int n_sel, int n_sink, int base_chunk,
                                                    int first_new_chunk, int n_new)
{
    __shared__ int found_at;
    int32_t *list = chunk_idx + (int64_t)blockIdx.x * n_sel;
    for (int c = first_new_chunk; c < first_new_chunk + n_new; ++c) {
        if (threadIdx.x == 0) found_at = -1;
        __syncthreads();
        for (int j = threadIdx.x; j < n_sel; j += 256)
            if (list[j] == c) found_at = j;          // the list holds no chunk twice: at most one writer
        __syncthreads();
        if (threadIdx.x == 0) {
            const int pos = n_sel - 1 - (c - base_chunk);
            const int j = found_at;
            if (j < 0) {
                list[pos] = c;                        // evicts the least important entry still listed
            } else if (j >= n_sink && j != pos) {     // already listed: trade places, nothing is evicted
                list[j] = list[pos];
                list[pos] = c;
            }
        }
        __syncthreads();
    }
}

// ---- copy the listed chunks into contiguous buffers ----------------------------------------------
// grid (n_sel * chunk_size / 16, n_kv_heads), 256 threads: one 16-lane group per row, 16 rows
// per workgroup; K then V.
__global__ void __launch_bounds__(256) gather_kernel(const GatherParams p)
{
    const int tid = threadIdx.x;
    const int c = tid & 15;
    const int h = blockIdx.y;
    const int64_t out_row = (int64_t)blockIdx.x * 16 + (tid >> 4);      // row of the gathered buffer
    const int sel = (int)(out_row / p.chunk_size);
    const int within = (int)(out_row - (int64_t)sel * p.chunk_size);
    const int64_t t = (int64_t)p.chunk_idx[(int64_t)h * p.n_sel + sel] * p.chunk_size + within;
    const bool valid = t >= 0 && t < p.n_tokens;
    u32x4 kr = {0u, 0u, 0u, 0u}, vr = {0u, 0u, 0u, 0u};
    if (valid) {
        const int64_t off = (int64_t)h * p.stride_head + t * p.stride_token + c * 8;
        kr = load_stream(p.k + off);
        vr = load_stream(p.v + off);
    }
    const int64_t o = ((int64_t)h * p.n_sel * p.chunk_size + out_row) * kHeadDim + c * 8;
    *reinterpret_cast<u32x4 *>(p.k_out + o) = kr;
    *reinterpret_cast<u32x4 *>(p.v_out + o) = vr;
}

// ---- per-chunk key sums ---------------------------------------------------------------------------
// One wavefront per chunk: lane = (row mod 4, 16-byte slice); 16 rows in flight per lane; the
// four row groups are summed across the wavefront and lanes 0..15 write the 128 sums.
__global__ void __launch_bounds__(256) ksum_kernel(const KsumParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int c = lane & 15, r = lane >> 4;
    const int64_t chunk = p.chunk_begin + (int64_t)blockIdx.x * 4 + wave;
    const int h = blockIdx.y;
    if (chunk >= p.chunk_end) return;
    const int64_t t_begin = chunk * p.chunk_size;
    int64_t t_end = t_begin + p.chunk_size;
    if (t_end > p.n_tokens) t_end = p.n_tokens;

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
#pragma unroll
    for (int x = 0; x < 8; ++x) ksum[x] = xrow_sum(ksum[x]);
    if (r == 0) {
        float *dst = p.ksum + (int64_t)h * p.ksum_stride_head + chunk * kHeadDim + c * 8;
        __builtin_nontemporal_store(f32x4{ksum[0], ksum[1], ksum[2], ksum[3]}, reinterpret_cast<f32x4 *>(dst));
        __builtin_nontemporal_store(f32x4{ksum[4], ksum[5], ksum[6], ksum[7]}, reinterpret_cast<f32x4 *>(dst + 4));
    }
}

// ---- chunk scores from the key sums ------------------------------------------------------------------
// A 16-lane group owns one chunk at a time (8 dimensions per lane, two 128-bit loads); a
// wavefront covers 16 chunks, all of its loads issued before the first use.
template <int G>
__global__ void __launch_bounds__(256) scores_from_sums_kernel(const SumScoresParams p)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int c = lane & 15, r = lane >> 4;
    const int h = blockIdx.y;
    const int64_t chunk0 = ((int64_t)blockIdx.x * 4 + wave) * 16;
    if (chunk0 >= p.n_chunks) return;
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
    const float *base = p.ksum + (int64_t)h * p.ksum_stride_head + c * 8;
    f32x4 a[4], b[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t chunk = chunk0 + i * 4 + r;
        const f32x4 z = {0.f, 0.f, 0.f, 0.f};
        a[i] = chunk < p.n_chunks ? *reinterpret_cast<const f32x4 *>(base + chunk * kHeadDim) : z;
        b[i] = chunk < p.n_chunks ? *reinterpret_cast<const f32x4 *>(base + chunk * kHeadDim + 4) : z;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int64_t chunk = chunk0 + i * 4 + r;
        float d = 0.f;
#pragma unroll
        for (int x = 0; x < 4; ++x) d = fmaf(qbar[x], a[i][x], fmaf(qbar[4 + x], b[i][x], d));
        d = row16_sum(d);
        int64_t count = p.n_tokens - chunk * p.chunk_size;
        if (count > p.chunk_size) count = p.chunk_size;
        if (c == 0 && chunk < p.n_chunks) p.scores[(int64_t)h * p.n_chunks + chunk] = p.scale * d / (float)count;
    }
}

template <int G>
hipError_t launch_sum_scores_g(const SumScoresParams &p, hipStream_t stream)
{
    dim3 grid((unsigned)((p.n_chunks + 63) / 64), p.n_kv_heads);
    hipLaunchKernelGGL(scores_from_sums_kernel<G>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_append(const AppendParams &p, hipStream_t stream)
{
    hipLaunchKernelGGL(append_kernel, dim3(p.n_accepted, p.n_kv_heads), dim3(64), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_admit(int32_t *chunk_idx, int n_kv_heads, int n_sel, int n_sink, int base_chunk, int first_new_chunk, int n_new,
                        hipStream_t stream)
{
    hipLaunchKernelGGL(admit_kernel, dim3(n_kv_heads), dim3(256), 0, stream, chunk_idx, n_sel, n_sink, base_chunk, first_new_chunk, n_new);
    return hipGetLastError();
}

hipError_t launch_gather(const GatherParams &p, hipStream_t stream)
{
    dim3 grid((unsigned)((int64_t)p.n_sel * p.chunk_size / 16), p.n_kv_heads);
    hipLaunchKernelGGL(gather_kernel, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_ksum(const KsumParams &p, hipStream_t stream)
{
    dim3 grid((unsigned)((p.chunk_end - p.chunk_begin + 3) / 4), p.n_kv_heads);
    hipLaunchKernelGGL(ksum_kernel, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

hipError_t launch_sum_scores(const SumScoresParams &p, hipStream_t stream)
{
    switch (p.group) {
        case 1: return launch_sum_scores_g<1>(p, stream);
        case 2: return launch_sum_scores_g<2>(p, stream);
        case 3: return launch_sum_scores_g<3>(p, stream);
        case 4: return launch_sum_scores_g<4>(p, stream);
        case 5: return launch_sum_scores_g<5>(p, stream);
        case 6: return launch_sum_scores_g<6>(p, stream);
        case 7: return launch_sum_scores_g<7>(p, stream);
        case 8: return launch_sum_scores_g<8>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ts
