// Top-k chunk selection for the partial cache (Alg. 1: C_p = first |S| entries plus the
// |B|-|S| most important others, from most to least important, Sec. 3.3), for gfx950.
//
// One workgroup per KV head.  Every candidate chunk gets a 64-bit key: high word = its score
// mapped to an unsigned integer that orders like the float (NaN lowest, -0 == +0), low word =
// ~index, so keys are distinct and "larger key" means "higher score, then lower index".
// Selecting k of n with k << n does not need a sort of all n:
//   1. radix select, up to 11 bits per pass from the top: a 2048-bin LDS histogram of the
//      candidates that still match the decided prefix, scanned from the top bin down, fixes the
//      next digit of the k-th largest key.  Digits that are the same for all keys (the upper
//      bits of ~index) are skipped: 3 passes for the score + 1..2 for the index at most.
//      The passes stop as soon as the keys from the chosen bin upwards fit the ordering step
//      (usually after the first pass; none is needed when all candidates fit), which then makes
//      the cut itself;
//   2. those keys (k or a few more) are compacted into LDS (slot order is arbitrary);
//   3. they are put in order and the first k are written: by rank counting (k <= 256: each key
//      counts the larger ones, several threads per key) or by a bitonic network in LDS (larger k).
// The step is a chain of short dependent phases, so what counts is the latency of each: up to
// 8192 candidates live in registers (8 per thread) instead of being re-read every pass, the
// histogram scan is a DPP prefix sum per wavefront plus one exchange of the wavefronts' totals,
// and every phase uses all wavefronts of the workgroup.
// The result does not depend on the arbitrary slot order, so the same call is bit-identical
// every time.  Bytes are negligible (4 per chunk): this step is latency, not bandwidth.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

constexpr int kRankCountMax = 256;     // most keys ordered by rank counting
constexpr int kRankAllMax = 192;       // up to here ranking all candidates costs less than one selection pass first
constexpr int kRegKeysMax = 8192;      // candidates held in registers: 8 per thread of 1024
constexpr int kBins = 2048;
constexpr int kHistBytes = kBins * 4;
constexpr int kCtlBytes = 16 + 16 * 4;   // control words, then the wavefronts' totals of the scan

__device__ __forceinline__ uint32_t order_key(float s)
{
    uint32_t u = __float_as_uint(s);
    if ((u & 0x7fffffffu) > 0x7f800000u) return 0u;   // NaN ranks below everything
    if (u == 0x80000000u) u = 0u;                     // -0 ranks with +0
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// inclusive prefix sum over the 64 lanes: shifts inside each 16-lane row by DPP, then the totals of
// the rows before this one
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_shr(uint32_t x)
{
    return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)x, CTRL, 0xf, 0xf, true);   // lanes shifted in from outside the row read 0
}
__device__ __forceinline__ uint32_t wave_inclusive_sum(uint32_t x, int lane)
{
    x += dpp_shr<0x111>(x);   // row_shr:1
    x += dpp_shr<0x112>(x);   // row_shr:2
    x += dpp_shr<0x114>(x);   // row_shr:4
    x += dpp_shr<0x118>(x);   // row_shr:8
    const uint32_t t0 = (uint32_t)__builtin_amdgcn_readlane((int)x, 15);
    const uint32_t t1 = (uint32_t)__builtin_amdgcn_readlane((int)x, 31);
    const uint32_t t2 = (uint32_t)__builtin_amdgcn_readlane((int)x, 47);
    const int row = lane >> 4;
    return x + (row >= 1 ? t0 : 0u) + (row >= 2 ? t1 : 0u) + (row >= 3 ? t2 : 0u);
}

// KPT: candidates per thread kept in registers (candidate tid + j*blockDim.x in slot j); 0 = too many
// for that, they are re-read from memory in every phase.
// n_sort: power of two >= k (size of the bitonic network; unused when k <= kRankCountMax)
// idx_bits: bits of the low word that can differ between keys (covers n_chunks - 1)
template <int KPT>
__global__ void __launch_bounds__(1024) topk_kernel(const TopkParams p, int n_sort, int idx_bits)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char lds_raw[];
    uint32_t *hist = reinterpret_cast<uint32_t *>(lds_raw);               // the bins; later the ranks of step 3
    uint32_t *ctl = reinterpret_cast<uint32_t *>(lds_raw + kHistBytes);   // [0] digit, [1] remaining k, [2] slot counter, [3] size of the chosen bin
    uint32_t *wtot = ctl + 4;
    uint64_t *sel = reinterpret_cast<uint64_t *>(lds_raw + kHistBytes + kCtlBytes);

    const int h = blockIdx.x;
    const int tid = threadIdx.x, nt = blockDim.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n_cand = p.n_chunks - p.n_sink;
    const float *s = p.scores + (int64_t)h * p.n_chunks + p.n_sink;
    int32_t *out = p.idx_out + (int64_t)h * (p.n_sink + p.k);

    for (int i = tid; i < p.n_sink; i += nt) out[i] = i;
    if (p.k == 0) return;

    uint32_t reg_key[KPT > 0 ? KPT : 1];
#pragma unroll
    for (int j = 0; j < KPT; ++j) {
        const int i = tid + j * nt;
        reg_key[j] = i < n_cand ? order_key(s[i]) : 0u;
    }
    // f(key) for every candidate of this thread
    auto for_each_key = [&](auto f) {
        if constexpr (KPT > 0) {
#pragma unroll
            for (int j = 0; j < KPT; ++j) {
                const int i = tid + j * nt;
                if (i < n_cand) f(((uint64_t)reg_key[j] << 32) | (uint64_t)(0xffffffffu - (uint32_t)(p.n_sink + i)));
            }
        } else {
            for (int i = tid; i < n_cand; i += nt) f(((uint64_t)order_key(s[i]) << 32) | (uint64_t)(0xffffffffu - (uint32_t)(p.n_sink + i)));
        }
    };
    if (tid == 0) ctl[2] = 0u;

    // ---- 1. radix select of the k-th largest key ---------------------------------------------
    const bool by_rank = p.k <= kRankCountMax;
    const uint32_t sel_cap = by_rank ? (uint32_t)kRankCountMax : (uint32_t)n_sort;   // keys the ordering step can take
    uint64_t prefix = 0ull, mask = 0ull;
    uint32_t kk = (uint32_t)p.k, n_sel = 0u;
    const int per = kBins / nt;                       // bins per thread of the scan: 8 (256 threads) or 2 (1024)
    const int n_idx_pass = idx_bits > 11 ? 2 : 1;
    // when all candidates fit the ordering step there is nothing to select first
    if ((uint32_t)n_cand <= (by_rank ? (uint32_t)kRankAllMax : sel_cap)) {
        n_sel = (uint32_t)n_cand;
        __syncthreads();   // the slot counter is cleared before the first slot is taken
    }
    for (int pass = 0; n_sel == 0u && pass < 3 + n_idx_pass; ++pass) {
        // score digits: bits 63..53, 52..42, 41..32; index digits: what idx_bits needs, 11 bits at most each
        int shift, width;
        if (pass < 3) shift = pass == 0 ? 53 : (pass == 1 ? 42 : 32), width = pass == 2 ? 10 : 11;
        else if (n_idx_pass == 2 && pass == 3) shift = 11, width = idx_bits - 11;
        else shift = 0, width = idx_bits < 11 ? idx_bits : 11;
        const uint32_t digit_mask = (1u << width) - 1u;
        for (int i = tid; i < kBins; i += nt) hist[i] = 0u;
        __syncthreads();
        for_each_key([&](uint64_t key) {
            if ((key & mask) == prefix) atomicAdd(&hist[(uint32_t)(key >> shift) & digit_mask], 1u);
        });
        __syncthreads();
        {
            // thread t owns bins kBins-1-per*t .. kBins-per-per*t (descending); find the bin where the
            // count of keys above it is < kk <= that count plus the bin's own
            uint32_t c[8], tot = 0u;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                c[j] = j < per ? hist[kBins - 1 - (per * tid + j)] : 0u;
                tot += c[j];
            }
            const uint32_t incl = wave_inclusive_sum(tot, lane);
            if (lane == 63) wtot[wave] = incl;
            __syncthreads();
            uint32_t above = incl - tot;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const uint32_t t = wtot[i];           // entries of wavefronts that do not exist are never added
                above += i < wave ? t : 0u;
            }
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                if (j < per && above < kk && kk <= above + c[j]) {
                    ctl[0] = (uint32_t)(kBins - 1 - (per * tid + j));
                    ctl[1] = kk - above;
                    ctl[3] = c[j];
                }
                above += c[j];
            }
        }
        __syncthreads();
        prefix |= (uint64_t)ctl[0] << shift;
        mask |= (uint64_t)digit_mask << shift;
        kk = ctl[1];
        // Keys above the chosen bin are wanted, keys below it are not, and the bin holds the cut.
        // Once everything from the bin upwards fits the ordering step, that step makes the cut
        // itself (it ranks the keys, and only the first k ranks are written): the remaining
        // digits need not be examined.  That is the case at the latest when the bin holds exactly
        // the keys still wanted.
        const uint32_t from_bin_up = (uint32_t)p.k - kk + ctl[3];
        if (from_bin_up <= sel_cap) n_sel = from_bin_up;
    }

    // ---- 2. compact the n_sel >= k keys from the chosen bin upwards ---------------------------------
    if (by_rank)
        for (int i = tid; i < (int)n_sel; i += nt) hist[i] = 0u;   // the ranks of step 3 (every thread is past its last read of the bins)
    for_each_key([&](uint64_t key) {
        if ((key & mask) >= prefix) {
            const uint32_t slot = atomicAdd(&ctl[2], 1u);
            if (slot < sel_cap) sel[slot] = key;   // always true: exactly n_sel keys qualify
        }
    });

    // ---- 3. order them, keep the first k ------------------------------------------------------------
    if (by_rank) {
        __syncthreads();
        // `parts` threads per key each count the larger keys in their share of the list and add
        // them up in LDS
        int parts = 1;
        while (parts < 16 && parts * 2 * (int)n_sel <= nt) parts *= 2;
        const int t = tid / parts, q = tid % parts;
        if (t < (int)n_sel) {
            const uint64_t mine = sel[t];
            uint32_t larger = 0u;
            int u = q;
            for (; u + 3 * parts < (int)n_sel; u += 4 * parts) {   // four independent reads in flight
                const uint64_t a0 = sel[u], a1 = sel[u + parts], a2 = sel[u + 2 * parts], a3 = sel[u + 3 * parts];
                larger += (a0 > mine ? 1u : 0u) + (a1 > mine ? 1u : 0u) + (a2 > mine ? 1u : 0u) + (a3 > mine ? 1u : 0u);
            }
            for (; u < (int)n_sel; u += parts) larger += (sel[u] > mine) ? 1u : 0u;
            if (larger) atomicAdd(&hist[t], larger);
        }
        __syncthreads();
        for (int t2 = tid; t2 < (int)n_sel; t2 += nt) {
            const uint32_t rank = hist[t2];
            if (rank < (uint32_t)p.k) out[p.n_sink + rank] = (int32_t)(0xffffffffu - (uint32_t)sel[t2]);
        }
        return;
    }
    for (int i = (int)n_sel + tid; i < n_sort; i += nt) sel[i] = 0ull;   // padding sorts last: real keys have a non-zero low word
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
    int idx_bits = 1;
    while (idx_bits < 32 && ((int64_t)1 << idx_bits) < (int64_t)p.n_chunks) ++idx_bits;
    const int nt = n_cand <= 64 ? 256 : 1024;
    const int per_thread = (n_cand + nt - 1) / nt;
    const size_t sel_cap = p.k > kRankCountMax ? (size_t)n_sort : (size_t)kRankCountMax;
    const size_t lds_bytes = kHistBytes + kCtlBytes + sel_cap * sizeof(uint64_t);
    auto launch = [&](auto kernel) {
        static std::atomic<uint64_t> lds_allowed{0};   // one per instantiation of this lambda, i.e. per kernel
        if (lds_bytes > 64 * 1024) {
            const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(kernel), 128 * 1024, lds_allowed);
            if (e != hipSuccess) return e;
        }
        hipLaunchKernelGGL(kernel, dim3(p.n_kv_heads), dim3(nt), lds_bytes, stream, p, n_sort, idx_bits);
        return hipGetLastError();
    };
    if (n_cand > kRegKeysMax) return launch(topk_kernel<0>);
    if (per_thread <= 1) return launch(topk_kernel<1>);
    if (per_thread <= 2) return launch(topk_kernel<2>);
    if (per_thread <= 4) return launch(topk_kernel<4>);
    return launch(topk_kernel<8>);
}

}  // namespace ts
