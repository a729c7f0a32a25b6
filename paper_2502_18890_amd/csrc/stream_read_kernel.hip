// Streaming-read probe: reads a device buffer once with 128-bit loads and folds it into one word.
// It does no useful work; the benchmark times it over the same cache buffers the attention passes
// read, which gives the read rate this chip actually sustains -- the practical ceiling that the
// HBM-bound passes (chunk scores, tree verification) can be compared with, next to the published
// peak.  Shape of the probe: many small workgroups, each reading one contiguous 32 KiB piece with
// eight independent 16-byte loads per lane in flight -- nothing but the memory system limits it.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

constexpr int kProbeVecPerWg = 2048;   // 16-byte vectors per workgroup: 32 KiB

__global__ void __launch_bounds__(256) stream_read_kernel(const u32x4 *__restrict__ src, int64_t n_vec, uint32_t *sink)
{
    const int64_t base = (int64_t)blockIdx.x * kProbeVecPerWg + threadIdx.x;
    u32x4 v[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int64_t j = base + i * 256;
        const u32x4 z = {0u, 0u, 0u, 0u};
        v[i] = j < n_vec ? __builtin_nontemporal_load(src + j) : z;
    }
    u32x4 acc = v[0];
#pragma unroll
    for (int i = 1; i < 8; ++i) acc ^= v[i];
    const uint32_t r = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
    // the store keeps the loads alive; it happens only for one value in 2^32, and then writes that value
    if (r == 0x5ca1ab1eu) *sink = r;
}

}  // namespace

hipError_t launch_stream_read(const void *src, int64_t n_vec, uint32_t *sink, hipStream_t stream)
{
    const int64_t n_wg = (n_vec + kProbeVecPerWg - 1) / kProbeVecPerWg;
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)n_wg), dim3(256), 0, stream, reinterpret_cast<const u32x4 *>(src), n_vec, sink);
    return hipGetLastError();
}

}  // namespace ts
