// Device-side helpers shared by the gfx950 kernels: vector types, bf16 handling,
// cross-lane reductions.  Wavefront size is 64 throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ts {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

constexpr int kHeadDim = 128;
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
// Finite stand-in for "no key seen yet": exp2(kNegBig - x) underflows to 0 and
// kNegBig - kNegBig is 0, so no NaN can arise from an all-masked tile.
constexpr float kNegBig = -1.0e30f;

__device__ __forceinline__ float bf16lo_to_f32(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16hi_to_f32(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// two floats -> packed bf16 pair (round to nearest even), first argument in the low half
__device__ __forceinline__ uint32_t pack_bf16(float a, float b)
{
    f32x2 x = {a, b};
    bf16x2 y = __builtin_convertvector(x, bf16x2);
    return __builtin_bit_cast(uint32_t, y);
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// ---- loads of data that a kernel reads exactly once ----------------------------------------------
// The cache rows are far larger than the on-die caches and every kernel here touches each of them
// once, so they are loaded with the non-temporal hint ("nt" on the instruction): a pure streaming
// read sustains 6.9 TB/s with it and 6.3 TB/s without on this chip.  The buffer loads that go straight
// to LDS carry the same hint through their cache-policy operand.
constexpr int kCachePolicyStream = 2;   // the "nt" bit of a buffer instruction's cache-policy operand
__device__ __forceinline__ u32x4 load_stream(const uint16_t *p)
{
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
}

// ---- reductions inside a group of 16 consecutive lanes (one DPP row) ----------------------
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xf, 0xf, true));
}
// After the call every lane of the 16-lane row holds the row's sum.
__device__ __forceinline__ float row16_sum(float x)
{
    x += dpp_mov<0xB1>(x);   // quad_perm [1,0,3,2]  : lane ^ 1
    x += dpp_mov<0x4E>(x);   // quad_perm [2,3,0,1]  : lane ^ 2
    x += dpp_mov<0x141>(x);  // row_half_mirror      : pairs the two quads of each 8 lanes
    x += dpp_mov<0x140>(x);  // row_mirror           : pairs the two halves of the row
    return x;
}

__device__ __forceinline__ float row16_max(float x)
{
    x = fmaxf(x, dpp_mov<0xB1>(x));
    x = fmaxf(x, dpp_mov<0x4E>(x));
    x = fmaxf(x, dpp_mov<0x141>(x));
    x = fmaxf(x, dpp_mov<0x140>(x));
    return x;
}

// ---- reductions across the four 16-lane rows of a wavefront (same lane%16) ----------------
// v_permlane16_swap exchanges odd rows of its first operand with even rows of its second,
// v_permlane32_swap the upper half of the first with the lower half of the second; applied
// to (x, x) each yields the two partners of a butterfly step.
__device__ __forceinline__ float xrow_max(float x)
{
    u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float xrow_sum(float x)
{
    u32x2 a = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    x = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// ---- coalesced write-back of an accumulator block through LDS --------------------------------
// A block of ROWS x 128 fp32 sits in LDS at `region`: row r at byte r*512, its 16-byte piece q at
// position q ^ (r & 31) (the owners of the accumulators write it that way, which keeps both their
// writes and these reads free of bank conflicts).  Rows [0, live_rows) go to dst (row pitch 128
// floats): 32 lanes cover one 512-byte row, so every store instruction writes two whole rows
// instead of 64 scattered 16-byte pieces.
template <int ROWS>
__device__ __forceinline__ void store_rows_from_lds(const unsigned char *region, int live_rows, float *dst, int lane)
{
    const int pc = lane & 31, half = lane >> 5;
#pragma unroll
    for (int r0 = 0; r0 < ROWS; r0 += 2) {
        const int r = r0 + half;
        const f32x4 v = *reinterpret_cast<const f32x4 *>(region + r * 512 + ((pc ^ (r & 31)) << 4));
        if (r < live_rows) __builtin_nontemporal_store(v, reinterpret_cast<f32x4 *>(dst + (int64_t)r * 128 + pc * 4));
    }
}

// full-wavefront sum, result in every lane
__device__ __forceinline__ float wave_sum(float x) { return xrow_sum(row16_sum(x)); }
__device__ __forceinline__ float wave_max(float x) { return xrow_max(row16_max(x)); }

}  // namespace ts
