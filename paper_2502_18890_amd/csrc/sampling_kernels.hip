// Penalized probabilities and pool sampling of TokenSwift (Sec. 3.4 "Contextual Penalty", Eq. 3;
// App. D: min-p, top-p and eta pools), for gfx950.  Rows are vocabulary-sized (32K..152K fp32): the
// probabilities pass is a split softmax bound by HBM (read the logits twice, write the
// probabilities once); the sampler works on one row per workgroup out of L2.
//
//   p_i = exp(l_i / (t * I_i)) / sum_j exp(l_j / (t * I_j)),  I_i = theta if token i is among the W
//   most recent generated tokens, else 1.
//
// Membership in the window: every workgroup builds the bitmap of its own 4096-entry slice in LDS
// from the list of recent token ids (a few KB, served by L2).  Arithmetic is fp32 in the exp2 domain.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

constexpr int kSlice = 4096;   // vocabulary entries per workgroup of the two softmax passes

// scaled logit in the exp2 domain: l * log2(e) / (t * I)
__device__ __forceinline__ float scaled_logit(float l, uint32_t word, int bit, float k_plain, float k_window)
{
    return l * (((word >> bit) & 1u) ? k_window : k_plain);
}

// One workgroup = one 4096-entry slice of one row.  PASS 0 writes the slice's (max, sum of
// exp2(x - max)); PASS 1 merges the row's slice statistics and writes the probabilities.
template <int PASS>
__global__ void __launch_bounds__(256) penalized_softmax_kernel(const PenaltyParams p)
{
    __shared__ float red[4];
    __shared__ uint32_t bits[kSlice / 32];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.y;
    const int64_t base = (int64_t)blockIdx.x * kSlice;
    const float *l = p.logits + (int64_t)row * p.vocab;

    if (tid < kSlice / 32) bits[tid] = 0u;
    __syncthreads();
    for (int i = tid; i < p.n_window; i += 256) {
        const int64_t off = (int64_t)p.window[i] - base;   // ids outside the vocabulary fall in no slice's live part
        if (off >= 0 && off < kSlice) atomicOr(&bits[off >> 5], 1u << (off & 31));
    }
    __syncthreads();

    const bool vec = (p.vocab % 4 == 0);   // rows stay 16-byte aligned: 128-bit accesses
    float x[16];
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int64_t i0 = base + it * 1024 + tid * 4;
        const uint32_t word = bits[(it * 1024 + tid * 4) >> 5];          // 4 consecutive ids share a word
        float lv[4] = {0.f, 0.f, 0.f, 0.f};
        if (vec && i0 + 3 < p.vocab) {
            const f32x4 q = *reinterpret_cast<const f32x4 *>(l + i0);
            lv[0] = q[0], lv[1] = q[1], lv[2] = q[2], lv[3] = q[3];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (i0 + e < p.vocab) lv[e] = l[i0 + e];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t i = i0 + e;
            x[it * 4 + e] = (i < p.vocab) ? scaled_logit(lv[e], word, (int)(i & 31), p.k_plain, p.k_window) : -INFINITY;
        }
    }

    if (PASS == 0) {
        float m = x[0];
#pragma unroll
        for (int e = 1; e < 16; ++e) m = fmaxf(m, x[e]);
        m = wave_max(m);
        if (lane == 0) red[wave] = m;
        __syncthreads();
        m = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
        __syncthreads();
        float s = 0.f;
#pragma unroll
        for (int e = 0; e < 16; ++e) s += fast_exp2(x[e] - m);   // exp2(-inf) = 0 for entries past the row
        s = wave_sum(s);
        if (lane == 0) red[wave] = s;
        __syncthreads();
        if (tid == 0) {
            float *st = p.stats + ((int64_t)row * p.n_slices + blockIdx.x) * 2;
            st[0] = m;
            st[1] = (red[0] + red[1]) + (red[2] + red[3]);
        }
        return;
    }

    // merge the slice statistics of the row (every workgroup of the row does the same, in the same order)
    const float *st = p.stats + (int64_t)row * p.n_slices * 2;
    float m_all = -INFINITY;
    for (int s = lane; s < p.n_slices; s += 64) m_all = fmaxf(m_all, st[2 * s]);
    m_all = wave_max(m_all);
    float z = 0.f;
    for (int s = lane; s < p.n_slices; s += 64) z += st[2 * s + 1] * fast_exp2(st[2 * s] - m_all);
    z = wave_sum(z);
    const float inv_z = 1.0f / z;
    float *out = p.probs + (int64_t)row * p.vocab;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
        const int64_t i0 = base + it * 1024 + tid * 4;
        if (vec && i0 + 3 < p.vocab) {
            f32x4 q;
#pragma unroll
            for (int e = 0; e < 4; ++e) q[e] = fast_exp2(x[it * 4 + e] - m_all) * inv_z;
            *reinterpret_cast<f32x4 *>(out + i0) = q;
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (i0 + e < p.vocab) out[i0 + e] = fast_exp2(x[it * 4 + e] - m_all) * inv_z;
        }
    }
}

// ---- pool sampling -------------------------------------------------------------------------------------
// One workgroup of 16 wavefronts per row.  Wavefront w owns the contiguous range [w*per, (w+1)*per) of
// the row and walks it in chunks of 256 entries (4 consecutive entries per lane), so "order of token
// id" = (wavefront, chunk, lane, entry).  All sums are taken in that fixed order: the same call is
// bit-identical every time.
struct RowWalker {
    const float *row;
    int64_t vocab, begin, end;   // this wavefront's range
    int lane;
    bool vec;                    // rows are 16-byte aligned: 128-bit loads

    __device__ __forceinline__ void load(int64_t c0, float (&v)[4]) const
    {
        const int64_t i0 = c0 + lane * 4;
        if (vec && i0 + 3 < end) {
            const f32x4 x = *reinterpret_cast<const f32x4 *>(row + i0);
            v[0] = x[0], v[1] = x[1], v[2] = x[2], v[3] = x[3];
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = (i0 + e < end) ? row[i0 + e] : 0.f;
        }
    }

    // f(chunk start, first entry of this lane, the lane's 4 entries), chunks in ascending order; four
    // chunks' loads are in flight at a time
    template <typename F>
    __device__ __forceinline__ void for_each_chunk(F f) const
    {
        int64_t c0 = begin;
        for (; c0 + 4 * 256 <= end; c0 += 4 * 256) {
            float v[4][4];
#pragma unroll
            for (int k = 0; k < 4; ++k) load(c0 + k * 256, v[k]);
#pragma unroll
            for (int k = 0; k < 4; ++k) f(c0 + k * 256, c0 + k * 256 + lane * 4, v[k]);
        }
        for (; c0 < end; c0 += 256) {
            float v[4];
            load(c0, v);
            f(c0, c0 + lane * 4, v);
        }
    }
};

__device__ __forceinline__ float block_sum16(float wave_total, float *red, int wave, int lane)
{
    __syncthreads();
    if (lane == 0) red[wave] = wave_total;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) s += red[w];
    return s;
}

// ---- top-p threshold ------------------------------------------------------------------------------------
// The pool of top-p is {v : p[v] >= tau} for the largest tau whose pool holds mass >= param.  Probabilities
// are non-negative floats, so their bit patterns order like their values and tau can be found digit by
// digit (11 + 11 + 9 bits of the pattern, three walks over the row): every entry that matches the digits
// decided so far adds its mass to the LDS bin of its next digit, and a scan from the top bin down finds the
// bin in which the running mass reaches what is still wanted.  Masses are added as integers (units of
// 2^-40, exact for p >= 2^-17, within half a unit below): integer sums do not depend on the order of the
// atomic adds, so the same call is bit-identical every time, and the decision differs from one taken on
// exact sums only when the mass at the cut is within vocab * 2^-41 of param.
constexpr int kMassBins = 2048;

__device__ __forceinline__ unsigned long long mass_units(float p)
{
    const float pc = fminf(p, 1.0f);
    const float hi = floorf(pc * 0x1p20f);             // exact: scaling by a power of two
    const float rem = fmaf(pc, 0x1p20f, -hi);          // exact, in [0, 1)
    const uint32_t lo = (uint32_t)fmaf(rem, 0x1p20f, 0.5f);
    return ((unsigned long long)(uint32_t)hi << 20) + lo;
}

__device__ float top_p_threshold(const RowWalker &w, float param, unsigned long long *hist, unsigned long long *wtot,
                                 unsigned long long *ctl, int tid)
{
    const int lane = tid & 63, wave = tid >> 6;
    unsigned long long want = (unsigned long long)ceil((double)param * 0x1p40);
    if (want == 0ull) want = 1ull;
    uint32_t prefix = 0u, mask = 0u;
#pragma unroll 1
    for (int level = 0; level < 3; ++level) {
        const int shift = level == 0 ? 20 : (level == 1 ? 9 : 0);
        const int n_bins = level == 2 ? 512 : 2048;
        for (int i = tid; i < n_bins; i += 1024) hist[i] = 0ull;
        if (tid == 0) ctl[0] = ~0ull;
        __syncthreads();
        w.for_each_chunk([&](int64_t, int64_t, const float (&v)[4]) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const uint32_t bits = __float_as_uint(v[e]);
                if (v[e] > 0.f && (bits & mask) == prefix) {      // false for NaN and for the zeros past the row
                    const unsigned long long units = mass_units(v[e]);
                    if (units != 0ull) atomicAdd(&hist[(bits >> shift) & (uint32_t)(n_bins - 1)], units);
                }
            }
        });
        __syncthreads();
        // thread t owns bins n_bins-1-2t and n_bins-2-2t (descending): running mass above each bin
        unsigned long long c[2] = {0ull, 0ull};
        if (2 * tid < n_bins) c[0] = hist[n_bins - 1 - 2 * tid], c[1] = hist[n_bins - 2 - 2 * tid];
        const unsigned long long tot = c[0] + c[1];
        unsigned long long incl = tot;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const unsigned long long up = __shfl_up(incl, d, 64);
            if (lane >= d) incl += up;
        }
        if (lane == 63) wtot[wave] = incl;
        __syncthreads();
        unsigned long long above = incl - tot;
        for (int i = 0; i < wave; ++i) above += wtot[i];
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if (above < want && want <= above + c[j]) {
                ctl[0] = (unsigned long long)(n_bins - 1 - 2 * tid - j);
                ctl[1] = want - above;
            }
            above += c[j];
        }
        __syncthreads();
        if (ctl[0] == ~0ull) return 0.f;    // the whole row holds less than param (only at the first level): every token is in the pool
        prefix |= (uint32_t)ctl[0] << shift;
        mask |= (uint32_t)(n_bins - 1) << shift;
        want = ctl[1];
        __syncthreads();                    // ctl and hist are rewritten by the next level
    }
    return __uint_as_float(prefix);
}

__global__ void __launch_bounds__(1024) sample_kernel(const SampleParams p)
{
    __shared__ float red[16];
    __shared__ int pick;
    __shared__ unsigned long long hist[kMassBins], wtot[16], ctl[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = blockIdx.x;
    int64_t per = ((p.vocab + 15) / 16 + 255) / 256 * 256;   // whole chunks per wavefront
    RowWalker w;
    w.row = p.probs + (int64_t)r * p.vocab;
    w.vocab = p.vocab;
    w.begin = (int64_t)wave * per;
    w.end = w.begin + per < p.vocab ? w.begin + per : p.vocab;
    if (w.begin > p.vocab) w.begin = p.vocab;
    w.lane = lane;
    w.vec = (p.vocab % 4 == 0) && ((reinterpret_cast<uintptr_t>(p.probs) & 15u) == 0);

    // ---- threshold of the pool -------------------------------------------------------------------
    float tau = 0.f;
    if (p.method == kSampleTopP) {
        tau = top_p_threshold(w, p.param, hist, wtot, ctl, tid);
    } else if (p.method != kSampleFull) {
        float m = 0.f;
        w.for_each_chunk([&](int64_t, int64_t, const float (&v)[4]) { m = fmaxf(fmaxf(m, fmaxf(v[0], v[1])), fmaxf(v[2], v[3])); });
        m = wave_max(m);
        __syncthreads();
        if (lane == 0) red[wave] = m;
        __syncthreads();
        float p_max = 0.f;
#pragma unroll
        for (int i = 0; i < 16; ++i) p_max = fmaxf(p_max, red[i]);
        if (p.method == kSampleMinP) {
            tau = p.param * p_max;
        } else if (p.method == kSampleEta) {
            // eta = min(epsilon, alpha * exp(-h)), h = -sum p ln p
            float hs = 0.f;
            w.for_each_chunk([&](int64_t, int64_t, const float (&v)[4]) {
#pragma unroll
                for (int e = 0; e < 4; ++e) hs += (v[e] > 0.f) ? v[e] * fast_log2(v[e]) : 0.f;
            });
            const float h = -kLn2 * block_sum16(wave_sum(hs), red, wave, lane);
            tau = fminf(p.param, p.param2 * fast_exp2(-h * kLog2e));
        }
    }

    // ---- draw: invert the pool's cumulative distribution at u ------------------------------------------
    float mine = 0.f;
    w.for_each_chunk([&](int64_t, int64_t, const float (&v)[4]) {
#pragma unroll
        for (int e = 0; e < 4; ++e) mine += (v[e] >= tau) ? v[e] : 0.f;
    });
    mine = wave_sum(mine);
    const float total = block_sum16(mine, red, wave, lane);
    float u = p.u[r];
    u = fminf(fmaxf(u, 0.f), 0.99999994f);
    const float target = u * total;
    // the wavefront whose range holds the target (the last one with any mass if rounding overshoots)
    float before = 0.f;
    int owner = -1, last_with_mass = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        if (red[i] > 0.f) last_with_mass = i;
        if (owner < 0 && target < before + red[i]) owner = i;
        if (owner < 0) before += red[i];
    }
    if (owner < 0) {
        owner = last_with_mass;
        before = 0.f;
        for (int i = 0; i < owner; ++i) before += red[i];
    }
    if (tid == 0) pick = -1;
    __syncthreads();
    if (wave == owner) {
        float run = before;   // pool mass before the current chunk
        int found = -1, last_pool = -1;
        w.for_each_chunk([&](int64_t, int64_t i0, const float (&v)[4]) {
            float q[4], s = 0.f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                q[e] = (v[e] >= tau && i0 + e < w.end) ? v[e] : 0.f;
                s += q[e];
            }
            // inclusive scan of the lanes' sums
            float incl = s;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const float up = __shfl_up(incl, d, 64);
                if (lane >= d) incl += up;
            }
            float c = run + incl - s;   // pool mass before this lane's first entry
            int cand = -1, lastp = -1;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (q[e] > 0.f || (v[e] >= tau && i0 + e < w.end)) lastp = (int)(i0 + e);
                c += q[e];
                if (cand < 0 && q[e] > 0.f && target < c) cand = (int)(i0 + e);
            }
            // first lane with a candidate wins (lanes are in id order)
            const uint64_t has = __builtin_amdgcn_ballot_w64(cand >= 0);
            if (found < 0 && has != 0ull) found = __shfl(cand, __builtin_ctzll(has), 64);
            const uint64_t hasp = __builtin_amdgcn_ballot_w64(lastp >= 0);
            if (hasp != 0ull) last_pool = __shfl(lastp, 63 - __builtin_clzll(hasp), 64);
            run += __shfl(incl, 63, 64);
        });
        if (lane == 0) pick = found >= 0 ? found : last_pool;   // rounding pushed the target past the end: last pool token
    }
    __syncthreads();
    if (tid == 0) {
        p.tokens[r] = pick;
        if (p.pool_threshold) p.pool_threshold[r] = tau;
        if (p.pool_mass) p.pool_mass[r] = total;
    }
}

}  // namespace

hipError_t launch_penalized_probs(const PenaltyParams &p, hipStream_t stream)
{
    dim3 grid(p.n_slices, p.n_rows);
    hipLaunchKernelGGL(penalized_softmax_kernel<0>, grid, dim3(256), 0, stream, p);
    hipLaunchKernelGGL(penalized_softmax_kernel<1>, grid, dim3(256), 0, stream, p);
    return hipGetLastError();
}

int sampling_slices(int64_t vocab) { return (int)((vocab + kSlice - 1) / kSlice); }

hipError_t launch_sample(const SampleParams &p, hipStream_t stream)
{
    hipLaunchKernelGGL(sample_kernel, dim3(p.n_rows), dim3(1024), 0, stream, p);
    return hipGetLastError();
}

}  // namespace ts
