// Top-k chunk selection for the partial cache (Alg. 1: C_p = first |S| entries plus the
// |B|-|S| most important others, from most to least important, Sec. 3.3), for gfx950.
//
// One workgroup per KV head.  Every candidate chunk gets a 64-bit key: high word = its score
// mapped to an unsigned integer that orders like the float (NaN lowest, -0 == +0), low word =
// ~index, so keys are distinct and "larger key" means "higher score, then lower index".
// Selecting k of n with k << n does not need a sort of all n:
//   1. radix select, 8 bits per pass from the top: a 256-bin LDS histogram of the candidates
//      that still match the decided prefix, one wavefront scans it from the top bin down and
//      fixes the next digit of the k-th largest key.  Digits that are the same for all keys
//      (the upper bytes of ~index) are skipped: at most 4 passes for the score + 1..3 for the
//      index; the passes stop as soon as the bin of the k-th largest key holds exactly the
//      keys still wanted (typically after two or three digits of the score).
//   2. the k keys >= the k-th largest are compacted into LDS (slot order is arbitrary);
//   3. they are put in order: by rank counting (k <= 256: each key counts the larger ones,
//      all reads are LDS broadcasts) or by a bitonic network in LDS (larger k).
// The result does not depend on the arbitrary slot order, so the same call is bit-identical
// every time.  Bytes are negligible (4 per chunk): this step is latency, not bandwidth.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

constexpr int kRankCountMax = 256;     // largest k ordered by rank counting
constexpr int kStageKeysMax = 8192;    // candidates whose 32-bit score keys are staged in LDS
constexpr int kHistBytes = 256 * 4;
constexpr int kCtlBytes = 16;

__device__ __forceinline__ uint32_t order_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;   // NaN ranks below everything
    if (u == 0x80000000u) u = 0u;                     // -0 ranks with +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// n_sort: power of two >= k (size of the bitonic network; unused when k <= kRankCountMax)
// idx_bytes: bytes of the low word that can differ between keys (covers n_chunks - 1)
__global__ void __launch_bounds__(1024) topk_kernel(const TopkParams p, int n_sort, int idx_bytes, int stage_keys)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint32_t *hist = reinterpret_cast<uint32_t *>(lds_raw);
    uint32_t *ctl = reinterpret_cast<uint32_t *>(lds_raw + kHistBytes);   // [0] digit, [1] remaining k, [2] slot counter, [3] size of the chosen bin
    uint64_t *sel = reinterpret_cast<uint64_t *>(lds_raw + kHistBytes + kCtlBytes);
    const int sel_cap = p.k > kRankCountMax ? n_sort : p.k;
    uint32_t *skeys = reinterpret_cast<uint32_t *>(sel + sel_cap);

    const int h = blockIdx.x;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int n_cand = p.n_chunks - p.n_sink;
    const float *s = p.scores + (int64_t)h * p.n_chunks + p.n_sink;
    int32_t *out = p.idx_out + (int64_t)h * (p.n_sink + p.k);

    for (int i = tid; i < p.n_sink; i += nt) out[i] = i;
    if (p.k == 0) return;

    if (stage_keys)
        for (int i = tid; i < n_cand; i += nt) skeys[i] = order_key(s[i]);
    if (tid == 0) ctl[2] = 0u;
    auto key_of = [&](int i) -> uint64_t {
        const uint32_t hi = stage_keys ? skeys[i] : order_key(s[i]);
        return ((uint64_t)hi << 32) | (uint64_t)(0xffffffffu - (uint32_t)(p.n_sink + i));
    };

    // ---- 1. radix select of the k-th largest key ---------------------------------------------
    uint64_t prefix = 0ull, mask = 0ull;
    uint32_t kk = (uint32_t)p.k;
    const int n_pass = 4 + idx_bytes;
    for (int pass = 0; pass < n_pass; ++pass) {
        const int shift = pass < 4 ? 56 - 8 * pass : 8 * (idx_bytes - 1 - (pass - 4));
        for (int i = tid; i < 256; i += nt) hist[i] = 0u;
        __syncthreads();   // also orders the staging of skeys before its first use
        for (int i = tid; i < n_cand; i += nt) {
            const uint64_t key = key_of(i);
            if ((key & mask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < 64) {
            // lane l owns bins 255-4l .. 252-4l (descending); find the bin where the count of
            // keys above it is < kk <= that count plus the bin's own
            uint32_t c[4], tot = 0u;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                c[j] = hist[255 - (4 * tid + j)];
                tot += c[j];
            }
            uint32_t incl = tot;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t up = __shfl_up(incl, d, 64);
                if (tid >= d) incl += up;
            }
            uint32_t above = incl - tot;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (above < kk && kk <= above + c[j]) {
                    ctl[0] = (uint32_t)(255 - (4 * tid + j));
                    ctl[1] = kk - above;
                    ctl[3] = c[j];
                }
                above += c[j];
            }
        }
        __syncthreads();
        prefix |= (uint64_t)ctl[0] << shift;
        mask |= 0xffull << shift;
        kk = ctl[1];
        // Every key that shares the digits decided so far with the k-th largest is wanted: nothing
        // straddles the cut, so the remaining digits (of the score, and the index digits that
        // break ties) need not be examined.
        if (ctl[3] == kk) break;
    }

    // ---- 2. compact the k keys >= the k-th largest -------------------------------------------
    for (int i = tid; i < n_cand; i += nt) {
        const uint64_t key = key_of(i);
        if ((key & mask) >= prefix) {
            const uint32_t slot = atomicAdd(&ctl[2], 1u);
            if (slot < (uint32_t)p.k) sel[slot] = key;   // always true: exactly k keys qualify
        }
    }

    // ---- 3. order them -----------------------------------------------------------------------
    if (p.k <= kRankCountMax) {
        __syncthreads();
        for (int t = tid; t < p.k; t += nt) {
            const uint64_t mine = sel[t];
            int rank = 0;
            for (int u = 0; u < p.k; ++u) rank += (sel[u] > mine) ? 1 : 0;
            out[p.n_sink + rank] = (int32_t)(0xffffffffu - (uint32_t)mine);
        }
        return;
    }
    for (int i = p.k + tid; i < n_sort; i += nt) sel[i] = 0ull;   // padding sorts last: real keys have a non-zero low word
    __syncthreads();
    for (int kb = 2; kb <= n_sort; kb <<= 1) {
        for (int j = kb >> 1; j > 0; j >>= 1) {
            for (int i = tid; i < n_sort; i += nt) {
                const int l = i ^ j;
                if (l > i) {
                    const uint64_t a = sel[i], b = sel[l];
                    const bool descending = (i & kb) == 0;
                    if ((a < b) == descending) {
                        sel[i] = b;
                        sel[l] = a;
                    }
                }
            }
            __syncthreads();
        }
    }
    for (int i = tid; i < p.k; i += nt) out[p.n_sink + i] = (int32_t)(0xffffffffu - (uint32_t)sel[i]);
}

}  // namespace

hipError_t launch_topk(const TopkParams &p, hipStream_t stream)
{
    const int n_cand = p.n_chunks - p.n_sink;
    int n_sort = 2;
    while (n_sort < p.k) n_sort <<= 1;
    const int idx_bytes = p.n_chunks <= (1 << 8) ? 1 : (p.n_chunks <= (1 << 16) ? 2 : 3);
    const int stage_keys = n_cand <= kStageKeysMax ? 1 : 0;
    const int nt = n_cand <= 4096 ? 256 : 1024;
    const size_t sel_cap = p.k > kRankCountMax ? (size_t)n_sort : (size_t)p.k;
    const size_t lds_bytes = kHistBytes + kCtlBytes + sel_cap * sizeof(uint64_t) + (stage_keys ? (size_t)n_cand * sizeof(uint32_t) : 0);
    static std::atomic<uint64_t> lds_allowed{0};
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(topk_kernel), 128 * 1024, lds_allowed);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(topk_kernel, dim3(p.n_kv_heads), dim3(nt), lds_bytes, stream, p, n_sort, idx_bytes, stage_keys);
    return hipGetLastError();
}

}  // namespace ts
