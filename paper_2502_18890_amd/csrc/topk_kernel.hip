// Top-k chunk selection for the partial cache (Alg. 1: C_p = first |S| entries plus the
// |B|-|S| most important others, "ordered by decreasing importance", Sec. 3.3), for gfx950.
// One workgroup per KV head sorts all candidate chunks in LDS with a bitonic network on
// 64-bit keys: high word = the score mapped to an unsigned integer that orders like the
// float (NaN lowest, -0 == +0), low word = ~index, so a descending sort puts equal scores in
// ascending index order.  The number of chunks is small (<= 8192), so this is latency, not
// bandwidth.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

__device__ __forceinline__ uint32_t order_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;   // NaN ranks below everything
    if (u == 0x80000000u) u = 0u;                     // -0 ranks with +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__global__ void __launch_bounds__(1024) topk_kernel(const TopkParams p, int n_pow2)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint64_t *keys = reinterpret_cast<uint64_t *>(lds_raw);
    const int h = blockIdx.x;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int n_cand = p.n_chunks - p.n_sink;
    const float *s = p.scores + (int64_t)h * p.n_chunks;

    for (int i = tid; i < n_pow2; i += nt) {
        uint64_t key = 0ull;   // padding sorts last: every real key has a non-zero low word
        if (i < n_cand) {
            const uint32_t idx = (uint32_t)(p.n_sink + i);
            key = ((uint64_t)order_key(s[idx]) << 32) | (uint64_t)(0xffffffffu - idx);
        }
        keys[i] = key;
    }
    __syncthreads();
    for (int k = 2; k <= n_pow2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < n_pow2; i += nt) {
                const int l = i ^ j;
                if (l > i) {
                    const uint64_t a = keys[i], b = keys[l];
                    const bool descending = (i & k) == 0;
                    if ((a < b) == descending) {
                        keys[i] = b;
                        keys[l] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
    int32_t *out = p.idx_out + (int64_t)h * (p.n_sink + p.k);
    for (int i = tid; i < p.n_sink; i += nt) out[i] = i;
    for (int i = tid; i < p.k; i += nt) out[p.n_sink + i] = (int32_t)(0xffffffffu - (uint32_t)keys[i]);
}

}  // namespace

hipError_t launch_topk(const TopkParams &p, hipStream_t stream)
{
    int n_cand = p.n_chunks - p.n_sink;
    int n_pow2 = 2;
    while (n_pow2 < n_cand) n_pow2 <<= 1;
    int nt = n_pow2 / 2;
    if (nt < 64) nt = 64;
    if (nt > 1024) nt = 1024;
    hipLaunchKernelGGL(topk_kernel, dim3(p.n_kv_heads), dim3(nt), (size_t)n_pow2 * sizeof(uint64_t), stream, p, n_pow2);
    return hipGetLastError();
}

}  // namespace ts
