// Tree-masked verification attention over the full KV cache (Alg. 1 "Parallel Verification",
// App. E of the TokenSwift paper), split along the cache, for gfx950 -- the kernel for more than
// 32 query rows per KV head (GQA groups, wide trees), built on v_mfma_f32_32x32x16_bf16.
//
// On this part the 32x32x16 instruction delivers twice the flops per issue slot of 16x16x32,
// and once g*T reaches ~100 rows the pass is no longer HBM-bound: matrix cores, vector units and
// LDS are all busy and the chip lowers its clock (1.8 GHz measured under this kernel, 2.4 GHz
// under the 32-row one), so what counts is work per key, not the order it is issued in.  Work
// decomposition: one workgroup = one KV
// head x one contiguous range of cached tokens (split index n_split = the tree tokens with the
// ancestor mask) x up to 32*NRB*WR query rows; 32-row blocks are dealt round-robin to WR
// wavefronts, every wavefront applies a 32-key tile to its own blocks.  A workgroup may hold KG
// such sets of WR wavefronts ("key groups"): group g takes tiles g, g+KG, ... of the range with
// its own accumulators and the groups are merged through LDS at the end.  That puts KG
// wavefronts on every SIMD (more latency hiding, matrix and vector work of different tiles
// overlap) while the workgroup still writes a single partial and shares one copy of the query
// fragments.
//
//   S^T = K . Q^T    A = K tile  (32 keys x 16 dims),   B = Q^T (16 dims x 32 rows), 8 steps
//   O^T += V^T . P^T A = V^T     (32 cols x 16 keys),   B = P^T (16 keys x 32 rows), 2 steps x 4 column blocks
//
// Keys sit on the MFMA M axis, so the 16 logits a lane owns all belong to one query row (lane
// mod 32): running max and sum are per-lane state, the row max needs one v_permlane32_swap, and
// the probabilities a lane computes are exactly the B-operand elements it must supply for the
// second product (the contraction order of keys is permuted the same way on the V^T side).
// The V^T operand needs 8 keys of one column per lane while V sits key-major in LDS: that is what
// ds_read_b64_tr_b16 is for.  Within 16 lanes, source lane i points at 4 consecutive columns of
// one key and result lane j receives column j%4 of the sources 4r + j/4 (r = 0..3); with source
// i -> (key base + i/4, columns 4*(i%4)..) a result lane gets 4 consecutive keys of column j, and
// two such reads make one operand with no register shuffling.
// P is split into hi + lo (both bf16) and multiplied twice, which keeps ~16 bits per weight.
//
// Data path: buffer_load_dwordx4 ... lds moves four 256-byte rows per instruction from HBM
// straight into an NS-stage LDS ring (no VGPR staging); 16-byte pieces are permuted on the way
// in so that operand reads are bank-conflict free:
//   K rows: LDS piece pos of row R holds global piece pos ^ (R mod 16);
//   V rows: LDS piece pos of row R holds global piece pos ^ 4*(R mod 4)  (the four keys a
//           transposed read touches land in four different 64-byte bank groups).
// Rows past the end of a range are cut off by the buffer descriptor's byte count; the ring is
// cleared before a pass so a stage never holds anything but finite values (a masked key adds 0 * V).
#include <type_traits>
#include <utility>

#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

typedef __attribute__((address_space(3))) void *lds_void_ptr;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) const bf16x8 *lds_bf16x8_cptr;
typedef __attribute__((address_space(3))) u32x4 *lds_u32x4_ptr;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

constexpr int kTileKeys = 32;
constexpr int kStageBytes = kTileKeys * 512;   // K half then V half
constexpr int kVHalf = kTileKeys * 256;
constexpr int kQRowBytes = 272;                // padded query rows (QLDS)
constexpr float kRescaleSlack = 8.0f;          // log2 units
constexpr float kResidualShare = 1.0f / 8.0f;    // share of a row's running denominator from which a weight counts as concentrated
constexpr float kTinyShare = 1.0f / 1024.0f;    // a row whose largest output is below this share of its weight sum counts as too small for fp16 values
constexpr float kHalfShift = 6.0f;             // fp16 weights are taken 2^6 above the reference: at most 2^14, flushed below 2^-30 of that

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Largest of three by v_maximum3_f32 (NaN-propagating): written with fmaxf, every operand that comes out of a matrix
// instruction is first passed through a v_max_f32 x, x that quiets signalling NaNs, one more instruction per value.
// A NaN logit ends in a NaN weight either way.
__device__ __forceinline__ float max3(float a, float b, float c)
{
    return __builtin_elementwise_maximum(__builtin_elementwise_maximum(a, b), c);
}

__device__ __forceinline__ float swap32_max(float x)
{
    u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float swap32_sum(float x)
{
    u32x2 b = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// f(integral_constant<int, 0>), f(integral_constant<int, 1>), ... in order
template <int... I, class F>
__device__ __forceinline__ void for_each_index(std::integer_sequence<int, I...>, F &&f)
{
    (f(std::integral_constant<int, I>{}), ...);
}

// smallest divisor of 16 that is >= ceil(16 / wr): the first 16/LPW wavefronts of a key group issue
// LPW tile-load instructions each, the others none (so every wavefront's vmcnt arithmetic holds)
constexpr int loads_per_wave(int wr) { return wr >= 16 ? 1 : (wr >= 8 ? 2 : (wr >= 4 ? 4 : (wr >= 2 ? 8 : 16))); }

// NRB: 32-row blocks per wavefront; WR: wavefronts per key group (along the query rows); KG: key
// groups; NS: LDS stages per key group (one tile resident, two with HALF, the others in flight); OCC:
// wavefronts per SIMD the register budget is cut for; QLDS: query fragments live in LDS instead
// of registers; HALF: the second product runs in fp16 where the values allow it (see below).
//
// HALF.  With bf16 weights the second product needs two passes (weights and their rounding
// residuals) to stay inside the error bar; fp16 weights (11 bits) need one, a third less matrix
// work in a kernel whose clock is limited by power.  V is bf16 in HBM, so the value half of a tile
// is converted to fp16 in LDS, in place, one step before the tile is consumed (each wavefront
// converts a slice; two tiles are resident instead of one).  bf16 -> fp16 is exact for magnitudes
// in [2^-17, 65504] (down to 2^-14 as normal numbers, below that as subnormals whose spacing of 2^-24 still
// holds a bf16 value's eight bits).  Smaller ones keep an absolute error below 2^-25, harmless next to
// values of normal size; larger ones and NaN become infinity or NaN.  Whether that happened is read off the
// accumulators at the end of the pass (non-finite entries; rows whose whole output is tiny although
// non-zero values were converted): such a workgroup runs its range again with bf16 weights and
// residuals, so the result never depends on fp16's range, and workgroups that meet no such value pay
// two barriers and a scan of their accumulators for the check.
template <int NRB, int WR, int KG, int NS, int OCC, bool QLDS, bool HALF>
__global__ void __launch_bounds__(64 * WR * KG) __attribute__((amdgpu_waves_per_eu(OCC, OCC)))
verify_wide_kernel(const VerifyParams p)
{
    constexpr int NT = 64 * WR * KG;
    constexpr int LPW = loads_per_wave(WR);   // load instructions per loading wavefront per tile (16 x 1 KiB = one tile)
    static_assert(NS >= (HALF ? 3 : 2), "bad shape");
    static_assert((NS - 2) * LPW <= 63, "too many loads in flight for vmcnt");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave_id = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave = wave_id % WR;   // position along the query rows
    const int kg = wave_id / WR;     // key group
    const int n32 = lane & 31;     // query row within a 32-row block / key row of a K operand
    const int hh = lane >> 5;      // which half of the contraction slice this lane supplies
    const int j = lane & 15;       // 16-byte piece a lane moves in a tile load
    const int quad = lane >> 4;
    const int split = blockIdx.x;
    const int h = blockIdx.y;
    const bool is_tree = (split == p.n_split);

    const uint16_t *kbase, *vbase;
    int64_t tstride, t_begin, t_end;
    if (is_tree) {
        kbase = p.k_tree + (int64_t)h * kHeadDim;
        vbase = p.v_tree + (int64_t)h * kHeadDim;
        tstride = (int64_t)p.n_kv_heads * kHeadDim;
        t_begin = 0;
        t_end = p.n_tree;
    } else {
        kbase = p.k + (int64_t)h * p.stride_head;
        vbase = p.v + (int64_t)h * p.stride_head;
        tstride = p.stride_token;
        t_begin = (int64_t)split * p.split_len;
        t_end = t_begin + p.split_len < p.n_tokens ? t_begin + p.split_len : p.n_tokens;
    }
    // Positions inside the range are 32-bit offsets from its first token (a range is shorter than 2^31 tokens: the
    // host refuses longer caches), so that the per-step tests are scalar 32-bit compares.
    const int range_len = (int)(t_end - t_begin);

    // ---- rows of this wavefront: 32-row blocks wave, wave + WR, ... of the workgroup's row tile ----
    const int tile_row0 = blockIdx.z * p.rows_per_wg;
    const int tile_rows = (p.n_rows - tile_row0) < p.rows_per_wg ? (p.n_rows - tile_row0) : p.rows_per_wg;
    // number of live blocks of this wavefront (wave-uniform)
    const int n_blocks = (tile_rows + 31) >> 5;
    const int nrb_live = __builtin_amdgcn_readfirstlane(n_blocks > wave ? (n_blocks - wave + WR - 1) / WR : 0);

    // ---- query fragments (MFMA B operand): loads issued now, awaited after the prefetch is out --
    unsigned char *qlds = lds + KG * NS * kStageBytes + (wave * NRB * 32) * kQRowBytes;   // shared by the key groups
    u32x4 qraw[NRB][8];
    uint64_t amask_lo[NRB], amask_hi[NRB];   // ancestor-or-self bits of tree nodes 0..63 and 64..127
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int row = tile_row0 + (rb * WR + wave) * 32 + n32;
        const bool live = rb < nrb_live && row < p.n_rows;
        const int node = live ? row / p.group : 0;
        const int jj = live ? row % p.group : 0;
        const uint16_t *qrow = p.q + ((int64_t)node * p.n_q_heads + h * p.group + jj) * kHeadDim;
        amask_lo[rb] = live ? p.anc[node][0] : 0ull;
        amask_hi[rb] = live ? p.anc[node][1] : 0ull;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (live && (!QLDS || kg == 0)) raw = *reinterpret_cast<const u32x4 *>(qrow + ks * 16 + hh * 8);
            qraw[rb][ks] = raw;
        }
    }

    float m_run[NRB], l_run[NRB];
    float m_limit[NRB];   // (m_run + kRescaleSlack) in raw logit units: the largest raw logit the reference still covers
    const float inv_scale_log2 = 1.0f / p.scale_log2;
    f32x16 oacc[NRB][4];
    // ---- HBM -> LDS -------------------------------------------------------------------------
    // Load instruction ii (0..15) of a tile fills LDS block ii: K rows 4ii..4ii+3 for ii < 8,
    // V rows 4(ii-8).. for ii >= 8.  Wavefront `wave` of a key group issues ii = wave*LPW ..
    // wave*LPW+LPW-1 of that group's tiles if those are < 16, else nothing.  Group tile number u of
    // key group kg is tile u*KG + kg of the range and lives in stage kg*NS + u % NS.
    const bool loader = wave * LPW < 16;
    uint32_t goff[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int ii = wave * LPW + i;
        const int R = 4 * (ii & 7) + quad;                       // row of the tile this lane fetches from
        const int f = (ii >= 8) ? ((R & 3) << 2) : (R & 15);
        goff[i] = (uint32_t)(R * tstride * 2 + ((j ^ f) << 4));
    }
    // Tiles are issued and consumed strictly in order, so both sides keep running cursors (a few
    // scalar additions per step) instead of recomputing addresses from the tile number: the scalar
    // unit is shared by the whole CU and this code sits on every wavefront's path after the barrier.
    const uint32_t stage0 = kg * NS * kStageBytes;       // a key group's NS stages lie next to each other
    const uint32_t stage_end = stage0 + NS * kStageBytes;
    const int64_t tile_elems = (int64_t)KG * kTileKeys * tstride;      // elements between consecutive group tiles
    const uint16_t *kfill, *vfill;
    int fill_rel;              // offset in the range of the first row of the next tile to fill
    uint32_t fill_stage;
    uint32_t use_stage;        // stage of the group tile being consumed
    int rel_cur;               // offset in the range of its first token
    const uint32_t row_bytes = (uint32_t)(tstride * 2);   // <= 2^25
    auto issue_tile = [&]() {
        if (loader) {
            // bytes from the tile's first row up to the end of its last valid row (0: the tile lies past the range)
            const int rows = range_len - fill_rel;
            const uint32_t nrec = rows <= 0 ? 0u : (uint32_t)((rows < kTileKeys ? rows : kTileKeys) - 1) * row_bytes + 256u;
            const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(kfill), 0, nrec, 0x00020000);
            const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(vfill), 0, nrec, 0x00020000);
            unsigned char *stage = lds + fill_stage;
#pragma unroll
            for (int i = 0; i < LPW; ++i) {
                const int ii = wave * LPW + i;                       // wave-uniform
                const uint32_t go = goff[i];
                if (ii < 8)
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, (lds_void_ptr)(stage + ii * 1024), 16, go, 0, 0, kCachePolicyStream);
                else
                    __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lds_void_ptr)(stage + kVHalf + (ii - 8) * 1024), 16, go, 0, 0, kCachePolicyStream);
            }
            kfill += tile_elems;     // past the range the descriptor covers 0 bytes, so the base is never dereferenced
            vfill += tile_elems;
            fill_rel += KG * kTileKeys;
            fill_stage += kStageBytes;
            if (fill_stage >= stage_end) fill_stage = stage0;
        }
    };

    // per-lane LDS read offsets inside a stage
    int koff[8];   // K operand of step ks: key row n32, global piece 2ks+hh
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) koff[ks] = n32 * 256 + ((((ks << 1) | hh) ^ (n32 & 15)) << 4);
    // V (transposed reads): as a source, this lane points at key 4*hh + (lane%16)/4 of each group of
    // 8 keys and at columns 32*cb + 16*((lane/16)%2) + 4*(lane%4) .. +3
    int voff[4];
    {
        const int jb = lane & 15, i4 = jb >> 2, ilo = jb & 3, mh = (lane >> 4) & 1;
#pragma unroll
        for (int cb = 0; cb < 4; ++cb)
            voff[cb] = kVHalf + (4 * hh + i4) * 256 + ((4 * (cb ^ i4) + 2 * mh + (ilo >> 1)) << 4) + ((ilo & 1) << 3);
    }

    // Stage offsets as instruction immediates.  In the steady state of the main loop the stage a step reads is known at
    // compile time (the loop is unrolled NS times), so an LDS address is a loop-invariant register (LDS base, key group's
    // first stage, the lane's offset) plus an immediate, and the dozen address additions per step go away.  Possible
    // where the whole ring lies within the 16-bit offset field of a DS instruction.
    // (Not where registers are scarce: NS copies of the tile body keep more values alive, and the shapes cut for three
    // wavefronts per SIMD, or converting four pieces per lane, would spill.)
    constexpr bool kImmStages = NS * kStageBytes <= 65536 && OCC <= 2 && !(HALF && WR < 4);
    const uint32_t lds32 = (uint32_t)(uintptr_t)lds + stage0;   // low half of a generic LDS address = LDS offset
    uint32_t kaddr[8], vaddr[4];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) kaddr[ks] = lds32 + koff[ks];
#pragma unroll
    for (int cb = 0; cb < 4; ++cb) vaddr[cb] = lds32 + voff[cb];
    const uint32_t caddr = lds32 + kVHalf + (wave * 64 + lane) * 16;   // first 16-byte piece this lane converts

    const int n_tiles = (range_len + kTileKeys - 1) / kTileKeys;
    const int n_steps = (n_tiles + KG - 1) / KG;   // group tiles per key group (some groups may run one empty)
    // ---- start of a pass over the range (a workgroup makes one, or two if fp16 did not fit) ----
    constexpr int kLdsUsed = KG * NS * kStageBytes + (QLDS ? 32 * NRB * WR * kQRowBytes : 0);
    uint32_t *unfit_note = reinterpret_cast<uint32_t *>(lds + kLdsUsed);   // 16 bytes behind everything else
    auto pass_begin = [&](auto half_tag, bool first) {
        constexpr int RES = decltype(half_tag)::value ? 2 : 1;   // tiles resident in LDS while the others are in flight
        // clear the ring: a stage must never hold anything but finite values (a masked key adds
        // 0 * V), whatever an earlier pass or workgroup left there
        {
            const u32x4 z = {0u, 0u, 0u, 0u};
            for (int off = tid * 16; off < KG * NS * kStageBytes; off += NT * 16) *reinterpret_cast<u32x4 *>(lds + off) = z;
            if (first && tid == 0) *reinterpret_cast<u32x2 *>(unfit_note) = u32x2{0u, 0u};
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS traffic only
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            m_run[rb] = kNegBig;
            m_limit[rb] = kNegBig;   // any finite logit moves the reference
            l_run[rb] = 0.f;
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[rb][cb][e] = 0.f;
        }
        kfill = kbase + (t_begin + (int64_t)kg * kTileKeys) * tstride;
        vfill = vbase + (t_begin + (int64_t)kg * kTileKeys) * tstride;
        fill_rel = kg * kTileKeys;
        fill_stage = stage0;
        use_stage = stage0;
        rel_cur = kg * kTileKeys;
#pragma unroll
        for (int s = 0; s < NS - RES; ++s) issue_tile();   // tiles past the range load nothing but still count
    };
    if constexpr (HALF) pass_begin(std::true_type{}, true);
    else pass_begin(std::false_type{}, true);

    // Now wait for the query and mask loads (older than every tile load, so the tile loads stay
    // in flight) -- here, not at their first use inside the main loop, where the wait would be
    // for everything issued before it, i.e. for the whole prefetched ring.
    bf16x8 qf[QLDS ? 1 : NRB][8];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        asm volatile("" ::"v"(amask_lo[rb]), "v"(amask_hi[rb]));
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            asm volatile("" ::"v"(qraw[rb][ks]));
            if (QLDS) {   // written once, by key group 0; first read after the first barrier of the main loop
                if (kg == 0)
                    *reinterpret_cast<u32x4 *>(qlds + (rb * 32 + n32) * kQRowBytes + (ks * 16 + hh * 8) * 2) = qraw[rb][ks];
            } else
                qf[rb][ks] = __builtin_bit_cast(bf16x8, qraw[rb][ks]);
        }
    }
    if (QLDS) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // the fragments are in LDS before this wavefront reaches the first barrier

    // ---- fp16 pass: conversion of a landed tile's values ------------------------------------------
    // The value half of a landed tile goes from bf16 to fp16 in place, one step before the tile is
    // consumed; rows past the end of the range become zero (a masked key then adds 0 * 0).  The 512
    // 16-byte pieces of a tile are shared by the WR wavefronts of its key group, kConvPieces per lane.
    // The work is cut in three so that its arithmetic can sit between the matrix instructions of the
    // first product (a chain of eight dependent instructions that leaves the vector unit idle):
    // conv_load (LDS reads, issued with the key operands), conv_piece_dword (one 32-bit word: two
    // values), conv_store.
    constexpr int kConvPieces = (kTileKeys * 16 + WR * 64 - 1) / (WR * 64);
    u32x4 conv_raw[kConvPieces], conv_out[kConvPieces];
    uint32_t conv_seen = 0u;   // every bit that was set in any value this lane converted (zero: it saw nothing but zeros)
    // stage_tag: index of the stage within the key group's ring if known at compile time, else -1 (then `stage` is used)
    auto conv_load = [&](auto stage_tag, const unsigned char *stage) {
        constexpr int SI = decltype(stage_tag)::value;
#pragma unroll
        for (int i = 0; i < kConvPieces; ++i) {
            const int pc = wave * 64 + lane + i * WR * 64;
            const u32x4 z = {0u, 0u, 0u, 0u};
            if constexpr (SI >= 0)
                conv_raw[i] = pc < kTileKeys * 16 ? *reinterpret_cast<lds_u32x4_ptr>(caddr + (SI * kStageBytes + i * WR * 1024)) : z;
            else
                conv_raw[i] = pc < kTileKeys * 16 ? *reinterpret_cast<lds_u32x4_ptr>(caddr + ((uint32_t)(stage - lds) - stage0) + i * WR * 1024) : z;
        }
    };
    // word w of piece i: two values converted
    auto conv_piece_dword = [&](int i, int w) {
        const uint32_t x = conv_raw[i][w];
        const f32x2 two = {bf16lo_to_f32(x), bf16hi_to_f32(x)};
        conv_out[i][w] = __builtin_bit_cast(uint32_t, __builtin_convertvector(two, f16x2));
    };
    // rel: offset in the range of the tile's first token; full_tag: the tile is known to lie wholly inside the range
    // (the steady state of the main loop), so no row has to be blanked
    auto conv_store = [&](auto stage_tag, auto full_tag, unsigned char *stage, int rel) {
        constexpr int SI = decltype(stage_tag)::value;
        constexpr bool FULL = decltype(full_tag)::value;
        const int left = range_len - rel;
        const int n_valid = left < 0 ? 0 : (left > kTileKeys ? kTileKeys : left);   // wavefront-uniform
#pragma unroll
        for (int i = 0; i < kConvPieces; ++i) {
            const int pc = wave * 64 + lane + i * WR * 64;
            if (pc < kTileKeys * 16) {
                const bool valid = FULL || (pc >> 4) < n_valid;
                if (valid) conv_seen |= conv_raw[i][0] | conv_raw[i][1] | conv_raw[i][2] | conv_raw[i][3];
                const u32x4 z = {0u, 0u, 0u, 0u};
                const u32x4 val = valid ? conv_out[i] : z;
                if constexpr (SI >= 0) *reinterpret_cast<lds_u32x4_ptr>(caddr + (SI * kStageBytes + i * WR * 1024)) = val;
                else *reinterpret_cast<lds_u32x4_ptr>(caddr + ((uint32_t)(stage - lds) - stage0) + i * WR * 1024) = val;
            }
        }
    };
    // the whole conversion at once (first tile of a pass; wavefronts without live row blocks)
    auto convert_values = [&](unsigned char *stage, int rel) {
        conv_load(std::integral_constant<int, -1>{}, stage);
#pragma unroll
        for (int i = 0; i < kConvPieces; ++i)
#pragma unroll
            for (int w = 0; w < 4; ++w) conv_piece_dword(i, w);
        conv_store(std::integral_constant<int, -1>{}, std::false_type{}, stage, rel);
    };

    // One 32-key tile against all of this wavefront's row blocks.  RAGGED tiles (the last one of
    // a range, every tile of the tree split) mask keys; full tiles carry no masking code.
    // L = number of row blocks computed (compile time, so that the body is straight-line code the
    // scheduler can interleave freely); a block beyond the wavefront's live ones holds zero queries
    // and is never written back.

    // ---- S^T = K . Q^T of one tile --------------------------------------------------------------
    // conv_tag: also convert the values of the tile in conv_stage (first token conv_t0), between the products
    // stage_tag: index of the tile's stage in the ring when the caller knows it at compile time (then the next stage, the
    // one converted, is known too), else -1; conv_full_tag: the converted tile lies wholly inside the range
    auto qk_tile = [&](auto live_tag, auto conv_tag, auto conv_full_tag, auto stage_tag, const unsigned char *stage,
                       unsigned char *conv_stage, int conv_rel, auto &sacc) {
        constexpr int L = decltype(live_tag)::value;
        constexpr bool CONV = decltype(conv_tag)::value;
        constexpr int SI = decltype(stage_tag)::value;
        constexpr int SN = SI >= 0 ? (SI + 1) % NS : -1;
        const std::integral_constant<int, SN> next_tag{};
        const uint32_t stage_rel = (uint32_t)(stage - lds) - stage0;   // the stage's offset from the key group's first one (scalar)
#pragma unroll
        for (int rb = 0; rb < L; ++rb)
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[rb][e] = 0.f;
        // all eight key operands are requested before the first product, so that the chain of
        // matrix instructions waits for LDS once, not eight times
        bf16x8 ka[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if constexpr (SI >= 0) ka[ks] = *reinterpret_cast<lds_bf16x8_cptr>(kaddr[ks] + SI * kStageBytes);
            else ka[ks] = *reinterpret_cast<lds_bf16x8_cptr>(kaddr[ks] + stage_rel);
        }
        if constexpr (CONV) conv_load(next_tag, conv_stage);
        __builtin_amdgcn_sched_barrier(0);
        constexpr int kWords = 4 * kConvPieces;               // 32-bit words this lane converts
        constexpr int kPerSlot = (kWords + 7) / 8;            // ... per matrix instruction of the chain
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int rb = 0; rb < L; ++rb) {
                const bf16x8 b = QLDS ? *reinterpret_cast<const bf16x8 *>(
                                            qlds + (rb * 32 + n32) * kQRowBytes + (ks * 16 + hh * 8) * 2)
                                      : qf[QLDS ? 0 : rb][ks];
                sacc[rb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ka[ks], b, sacc[rb], 0, 0, 0);
            }
            if constexpr (CONV) {
#pragma unroll
                for (int c = ks * kPerSlot; c < (ks + 1) * kPerSlot && c < kWords; ++c) conv_piece_dword(c >> 2, c & 3);
            }
        }
        if constexpr (CONV) conv_store(next_tag, conv_full_tag, conv_stage, conv_rel);
    };

    // Tile sums for the chunk scores (see pv_tile).  The store of a tile's sum waits until just before
    // the next loads are issued: vmcnt counts loads and stores alike, in order, so a store younger than
    // the loads a step waits for would put its own latency on that wait.
    const bool scoring = p.tile_sums != nullptr && wave == 0 && blockIdx.z == 0 && !is_tree;   // wavefront-uniform
    float score_parked = 0.f;
    int score_parked_tile = -1;   // tile of the range (cache ranges begin on a tile boundary)
    float *const tile_sums_range = scoring ? p.tile_sums + (int64_t)h * p.tile_sums_stride + (t_begin >> 5) : nullptr;
    auto score_flush = [&]() {
        if (scoring && score_parked_tile >= 0) {
            if (lane == 0) tile_sums_range[score_parked_tile] = score_parked;
            score_parked_tile = -1;
        }
    };

    // ---- softmax of one tile's logits and O^T += V^T . P^T ----------------------------------------
    // RAGGED tiles (the last one of a range, every tile of the tree split) mask keys; full tiles
    // carry no masking code.
    auto pv_tile = [&](auto live_tag, auto ragged_tag, auto half_tag, auto stage_tag, const unsigned char *stage, int rel, auto &sacc) {
        constexpr int L = decltype(live_tag)::value;
        constexpr bool RAGGED = decltype(ragged_tag)::value;
        constexpr bool F16 = decltype(half_tag)::value;
        constexpr int SI = decltype(stage_tag)::value;

        // V^T operands: vt[cb][s] = column 32*cb + n32, keys 4*hh + 16*s + 8*(e/4) + e%4 (e = 0..7).
        // The sixteen transposed reads and their wait are one asm block: issued through the
        // compiler's builtin, each would be preceded by a wait for ALL outstanding tile loads
        // (LDS written by buffer_load ... lds is tracked by vmcnt and the builtin carries no alias
        // information), i.e. for the whole prefetched ring.  The stage read here was completed by
        // the vmcnt wait + barrier at the top of the step.  The block sits right behind the S^T
        // products, whose execution covers its LDS latency.
        bf16x8 vt[4][2];
        {
            constexpr int kImm = SI >= 0 ? SI * kStageBytes : 0;   // the stage's offset rides in the instructions
            uint32_t a0, a1, a2, a3;
            if constexpr (SI >= 0) {
                a0 = vaddr[0], a1 = vaddr[1], a2 = vaddr[2], a3 = vaddr[3];
            } else {
                const uint32_t stage_rel = (uint32_t)(stage - lds) - stage0;   // scalar
                a0 = vaddr[0] + stage_rel, a1 = vaddr[1] + stage_rel, a2 = vaddr[2] + stage_rel, a3 = vaddr[3] + stage_rel;
            }
            u32x2 r[16];
            asm volatile(
                "ds_read_b64_tr_b16 %0, %16 offset:%20\n\t"
                "ds_read_b64_tr_b16 %1, %16 offset:%21\n\t"
                "ds_read_b64_tr_b16 %2, %16 offset:%22\n\t"
                "ds_read_b64_tr_b16 %3, %16 offset:%23\n\t"
                "ds_read_b64_tr_b16 %4, %17 offset:%20\n\t"
                "ds_read_b64_tr_b16 %5, %17 offset:%21\n\t"
                "ds_read_b64_tr_b16 %6, %17 offset:%22\n\t"
                "ds_read_b64_tr_b16 %7, %17 offset:%23\n\t"
                "ds_read_b64_tr_b16 %8, %18 offset:%20\n\t"
                "ds_read_b64_tr_b16 %9, %18 offset:%21\n\t"
                "ds_read_b64_tr_b16 %10, %18 offset:%22\n\t"
                "ds_read_b64_tr_b16 %11, %18 offset:%23\n\t"
                "ds_read_b64_tr_b16 %12, %19 offset:%20\n\t"
                "ds_read_b64_tr_b16 %13, %19 offset:%21\n\t"
                "ds_read_b64_tr_b16 %14, %19 offset:%22\n\t"
                "ds_read_b64_tr_b16 %15, %19 offset:%23\n\t"
                "s_waitcnt lgkmcnt(0)"
                : "=&v"(r[0]), "=&v"(r[1]), "=&v"(r[2]), "=&v"(r[3]), "=&v"(r[4]), "=&v"(r[5]), "=&v"(r[6]), "=&v"(r[7]),
                  "=&v"(r[8]), "=&v"(r[9]), "=&v"(r[10]), "=&v"(r[11]), "=&v"(r[12]), "=&v"(r[13]), "=&v"(r[14]), "=&v"(r[15])
                : "v"(a0), "v"(a1), "v"(a2), "v"(a3), "n"(kImm), "n"(kImm + 2048), "n"(kImm + 4096), "n"(kImm + 6144)
                : "memory");
            // r[4*cb + 2*s + x]: keys 16*s + 8*x + 4*hh + (0..3) of column block cb
#pragma unroll
            for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    const u32x4 both = {r[4 * cb + 2 * s][0], r[4 * cb + 2 * s][1], r[4 * cb + 2 * s + 1][0], r[4 * cb + 2 * s + 1][1]};
                    vt[cb][s] = __builtin_bit_cast(bf16x8, both);
                }
        }

        // Chunk scores ride along: the rows of the first tree node (rows 0..group-1 of the first row block,
        // in wavefront 0 of every key group) hold exactly the raw logits q.k that Eq. 2 sums; their sum
        // over the tile's valid keys is parked until the next tile's loads are about to be issued (see
        // score_flush), and the merge kernel turns tiles into chunks.
        // (This lane's own sixteen logits are added here, while they are at hand; the cross-lane part of the sum waits
        // until the second product's matrix instructions have been issued and runs in their shadow.)
        const bool score_this = L > 0 && scoring && rel < range_len;
        float ssum = 0.f;
        if (score_this) {
            const uint32_t ok = RAGGED ? (uint32_t)((range_len - rel >= 32 ? 0xffffffffull : ((1ull << (range_len - rel)) - 1ull)) >> (hh * 4)) : 0xffffffffu;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const float v = sacc[0][e];
                ssum += (!RAGGED || ((ok >> (8 * (e >> 2) + (e & 3))) & 1u)) ? v : 0.f;
            }
        }

        // m_run is a reference point, not necessarily the exact running maximum: the accumulators are
        // rescaled only when a logit exceeds it by more than kRescaleSlack, so the weights stay
        // <= 2^kRescaleSlack and the (rare) rescale leaves the common path.  The common path only
        // compares each lane's largest raw logit (scale > 0 commutes with max) with m_limit, the same
        // bound in raw units; the row maximum across the two lanes of a row, the new reference and the
        // rescaling are the rare path's.  Element e of sacc is key hh*4 + 8*(e/4) + e%4 of the tile, for
        // query row n32.
        float mloc[L > 0 ? L : 1];
        bool moved = false;
#pragma unroll
        for (int rb = 0; rb < L; ++rb) {
            if (RAGGED) {
                uint64_t tile_ok;
                if (rel >= range_len) {   // a key group's tile past the end of the range: no keys
                    tile_ok = 0ull;
                } else if (is_tree) {     // the tree's range begins at node 0
                    const uint64_t w = (rel & 64) ? amask_hi[rb] : amask_lo[rb];
                    tile_ok = w >> (rel & 63);
                } else {
                    tile_ok = range_len - rel >= 64 ? ~0ull : ((1ull << (range_len - rel)) - 1ull);
                }
                const uint32_t vm = (uint32_t)tile_ok >> (hh * 4);
#pragma unroll
                for (int e = 0; e < 16; ++e)
                    if (!((vm >> (8 * (e >> 2) + (e & 3))) & 1u)) sacc[rb][e] = -INFINITY;
            }
            // three-input maxima: eight instructions for sixteen values
            float m = max3(sacc[rb][0], sacc[rb][1], sacc[rb][2]);
#pragma unroll
            for (int e = 3; e < 15; e += 2) m = max3(m, sacc[rb][e], sacc[rb][e + 1]);
            mloc[rb] = max3(m, sacc[rb][15], sacc[rb][15]);
            moved |= mloc[rb] > m_limit[rb];
        }
        if (__builtin_amdgcn_ballot_w64(moved) != 0ull) {   // some row of this wavefront outgrew its reference
#pragma unroll
            for (int rb = 0; rb < L; ++rb) {
                const float m_new = fmaxf(m_run[rb], swap32_max(mloc[rb]) * p.scale_log2);   // both lanes of a row agree on it
                const float alpha = fast_exp2(m_run[rb] - m_new);
                l_run[rb] *= alpha;
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) oacc[rb][cb][e] *= alpha;
                m_run[rb] = m_new;
                m_limit[rb] = (m_new + kRescaleSlack) * inv_scale_log2;
            }
        }

        // fp16 weights carry 11 bits.  That is enough where a row's weight is spread over many keys
        // (independent rounding errors of 2^-12 each), not where a few keys hold it: a tile in
        // which some lane's largest weight reaches kResidualShare of what that lane has accumulated
        // so far also multiplies the rounding residuals (fp16 again, 22 bits in all).  That second
        // product sits in a loop that runs zero or one times rather than in a branch:
        // accumulators updated inside an if get copied at the join, loop-carried ones stay put.
        int n_trips = 1;
        if constexpr (F16) {
            bool concentrated = false;
#pragma unroll
            for (int rb = 0; rb < L; ++rb)
                concentrated |= fast_exp2(fmaf(mloc[rb], p.scale_log2, kHalfShift - m_run[rb])) >= kResidualShare * l_run[rb];
            n_trips = __builtin_amdgcn_ballot_w64(concentrated) != 0ull ? 2 : 1;
        }

        // P = exp2(scale*s - m); O^T += V^T . P^T with P in fp16, or split hi + lo (both bf16)
#pragma unroll
        for (int rb = 0; rb < L; ++rb) {
            float pe[16], psum = 0.f;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                pe[e] = fast_exp2(fmaf(sacc[rb][e], p.scale_log2, (F16 ? kHalfShift : 0.f) - m_run[rb]));
                if constexpr (!F16) psum += pe[e];
            }
            if constexpr (F16) {
                // the row sum is taken over the weights as the matrix instruction sees them (rounded to fp16:
                // the normalisation then matches the product exactly), two per instruction
                f16x8 ph[2];
                const f16x2 ones = {(_Float16)1.0f, (_Float16)1.0f};
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    u32x4 w4;
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const f32x2 two = {pe[8 * s + 2 * w], pe[8 * s + 2 * w + 1]};
                        const f16x2 h2 = __builtin_convertvector(two, f16x2);
                        psum = __builtin_amdgcn_fdot2(h2, ones, psum, false);
                        w4[w] = __builtin_bit_cast(uint32_t, h2);
                    }
                    ph[s] = __builtin_bit_cast(f16x8, w4);
                }
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb)
                        oacc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, vt[cb][s]), ph[s], oacc[rb][cb], 0, 0, 0);
#pragma clang loop unroll(disable)
                for (int trip = 1; trip < n_trips; ++trip) {   // zero or one times
                    // weights of the second product: what rounding to fp16 left behind
#pragma unroll
                    for (int s = 0; s < 2; ++s) {
                        u32x4 w4;
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            // (halves taken as scalars: a bit_cast of one vector element to a
                            // two-element fp16 vector was seen compiled as element 0 for every w)
                            uint32_t had = __builtin_bit_cast(u32x4, ph[s])[w];
                            // the compiler must not compute these residuals ahead of the loop, on every tile
                            asm volatile("" : "+v"(had));
                            const float had_lo = (float)__builtin_bit_cast(_Float16, (uint16_t)(had & 0xffffu));
                            const float had_hi = (float)__builtin_bit_cast(_Float16, (uint16_t)(had >> 16));
                            const f32x2 left = {pe[8 * s + 2 * w] - had_lo, pe[8 * s + 2 * w + 1] - had_hi};
                            const f16x2 l2 = __builtin_convertvector(left, f16x2);
                            psum = __builtin_amdgcn_fdot2(l2, ones, psum, false);
                            w4[w] = __builtin_bit_cast(uint32_t, l2);
                        }
                        ph[s] = __builtin_bit_cast(f16x8, w4);
                    }
#pragma unroll
                    for (int s = 0; s < 2; ++s)
#pragma unroll
                        for (int cb = 0; cb < 4; ++cb)
                            oacc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, vt[cb][s]), ph[s], oacc[rb][cb], 0, 0, 0);
                }
                l_run[rb] += psum;
            } else {
                l_run[rb] += psum;
                bf16x8 p_hi[2], p_lo[2];
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    u32x4 hi, lo;
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const float a = pe[8 * s + 2 * w], b = pe[8 * s + 2 * w + 1];
                        const uint32_t hw = pack_bf16(a, b);
                        hi[w] = hw;
                        lo[w] = pack_bf16(a - bf16lo_to_f32(hw), b - bf16hi_to_f32(hw));
                    }
                    p_hi[s] = __builtin_bit_cast(bf16x8, hi);
                    p_lo[s] = __builtin_bit_cast(bf16x8, lo);
                }
#pragma unroll
                for (int s = 0; s < 2; ++s)
#pragma unroll
                    for (int cb = 0; cb < 4; ++cb) {
                        oacc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt[cb][s], p_hi[s], oacc[rb][cb], 0, 0, 0);
                        oacc[rb][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vt[cb][s], p_lo[s], oacc[rb][cb], 0, 0, 0);
                    }
            }
        }
        if (score_this) {
            ssum = swap32_sum(ssum);                                     // the two lanes that share row n32
            score_parked = row16_sum(n32 < p.group ? ssum : 0.f);       // the group's heads (group <= 8: one 16-lane row)
            score_parked_tile = rel >> 5;
        }
    };

    // Main loop over group tiles u = 0 .. n_steps-1 (tile u*KG + kg of the range): RES group tiles
    // resident, NS-RES in flight.  Every wavefront of the workgroup runs the same number of steps
    // (one barrier each), whichever instantiation of the body it takes.
    const int n_full_steps = is_tree ? 0 : (range_len / kTileKeys) / KG;   // steps whose tiles are full for every key group
    auto pass_main = [&](auto half_tag) {
        constexpr bool F16 = decltype(half_tag)::value;
        constexpr int RES = F16 ? 2 : 1;
        auto sync_and_refill = [&]() {
            // this wavefront's pieces of the next group tile have landed: the NS-RES-1 issued after
            // it may still be in flight
            // (a parked tile sum, stored just before the newest tile's loads were issued, is one more
            // operation allowed to be outstanding)
            if (scoring) wait_vmcnt<(NS - RES - 1) * LPW + (NS - RES - 1 > 0 ? 1 : 0)>();
            else wait_vmcnt<(NS - RES - 1) * LPW>();
            // ... and everyone's; all are done with the previous group tile.  A bare s_barrier:
            // __syncthreads() would add a fence that waits for every outstanding load, i.e. for the
            // whole prefetched ring.
            if (F16) asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wavefront's converted values are in LDS
            if (WR * KG > 1) asm volatile("s_barrier" ::: "memory");
            score_flush();
            issue_tile();                                          // refills the stage the previous group tile occupied
        };
        auto run = [&](auto live_tag) {
            constexpr int L = decltype(live_tag)::value;
            f32x16 s_cur[L > 0 ? L : 1];
            if (F16) {   // the first tile's values are converted before the loop; the barrier of step 0 publishes them
                sync_and_refill();
                convert_values(lds + use_stage, rel_cur);
            }
            // One step.  stage_tag: position of the tile's stage in the ring if the caller knows it at compile time (the
            // unrolled steady state), else -1 and the running use_stage is used; conv_full_tag: the tile after this one
            // (the one whose values are converted) lies wholly inside the range.
            auto step = [&](auto ragged_tag, auto conv_full_tag, auto stage_tag) {
                constexpr int SI = decltype(stage_tag)::value;
                sync_and_refill();
                // fp16: the tile after this one has landed too (two are resident); its values are converted
                // now, between the matrix instructions of this tile's first product
                uint32_t next_stage = use_stage + kStageBytes;
                if (next_stage >= stage_end) next_stage = stage0;
                if (L > 0) {
                    const unsigned char *stage = lds + use_stage;
                    qk_tile(live_tag, half_tag, conv_full_tag, stage_tag, stage, lds + next_stage, rel_cur + KG * kTileKeys, s_cur);
                    pv_tile(live_tag, ragged_tag, half_tag, stage_tag, stage, rel_cur, s_cur);
                } else if (F16) {
                    convert_values(lds + next_stage, rel_cur + KG * kTileKeys);
                }
                if constexpr (SI < 0) {     // (the unrolled loop leaves use_stage where it was: NS steps later)
                    use_stage += kStageBytes;
                    if (use_stage >= stage_end) use_stage = stage0;
                }
                rel_cur += KG * kTileKeys;
            };
            const std::integral_constant<int, -1> any_stage{};
            // Full tiles first, then the ragged end; the tree split is all ragged.  The steady state -- this tile and the
            // next both full -- runs NS steps per trip with the stages as compile-time constants.
            int u = 0;
            const int n_steady = F16 ? (n_full_steps > 0 ? n_full_steps - 1 : 0) : n_full_steps;
            if constexpr (kImmStages && L > 0) {
                for (; u + NS <= n_steady; u += NS) {
                    for_each_index(std::make_integer_sequence<int, NS>{},
                                   [&](auto stage_tag) { step(std::false_type{}, std::true_type{}, stage_tag); });
                }
            }
            for (; u < n_steady; ++u) step(std::false_type{}, std::true_type{}, any_stage);
            for (; u < n_full_steps; ++u) step(std::false_type{}, std::false_type{}, any_stage);
            for (; u < n_steps; ++u) step(std::true_type{}, std::false_type{}, any_stage);
        };
        if (nrb_live == NRB) run(std::integral_constant<int, NRB>{});
        else run(std::integral_constant<int, NRB - 1>{});   // round-robin dealing: never fewer than NRB-1 unless none at all
        score_flush();
        wait_vmcnt<0>();   // drain the loads issued past the range before LDS is reused or released
    };
    float m_shift = 0.f;   // how far above the reference point the weights of the pass that counts were taken
    if constexpr (HALF) {
        pass_main(std::true_type{});
        // Did fp16 hold the values of this range?  Judged from the result, once per pass: a value of 65520 or
        // more (or a NaN) became an infinity (NaN) in LDS and has made every accumulator of its column
        // non-finite, whatever its weight (0 * inf is NaN too); values below 2^-17 lost bits (2^-25 absolute at
        // most), which matters only where a row's whole output is that small: a row whose largest output
        // magnitude is below kTinyShare of its weight sum, although non-zero values were converted.
        if (__builtin_amdgcn_ballot_w64((conv_seen & 0x7fff7fffu) != 0u) != 0ull && lane == 0) unfit_note[1] = 1u;
        bool bad = false, tiny = false;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            if (rb < nrb_live) {
                float sum = 0.f, big = 0.f;
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const float a = fabsf(oacc[rb][cb][e]);
                        sum += a;                  // NaN and infinity survive a sum (a maximum would drop a NaN)
                        big = fmaxf(big, a);
                    }
                bad |= !(sum < 3.0e38f);
                const float l_tot = swap32_sum(l_run[rb]);
                tiny |= l_tot > 0.f && swap32_max(big) < kTinyShare * l_tot;
            }
        }
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        const bool seen = unfit_note[1] != 0u;
        if (__builtin_amdgcn_ballot_w64(bad || (seen && tiny)) != 0ull && lane == 0) unfit_note[0] = 1u;
        asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
        if (unfit_note[0] != 0u) {   // the same for every wavefront: run the range again with bf16 weights
            pass_begin(std::false_type{}, false);
            pass_main(std::false_type{});
        } else {
            m_shift = kHalfShift;
        }
    } else {
        pass_main(std::false_type{});
    }

    // ---- merge the key groups: groups 1.. hand (m, l, O) to group 0 through LDS ----------------
    // Each lane parks exactly the accumulator elements that the lane with the same position in
    // group 0 owns, so the exchange is lane-to-lane (no transposition); 16-byte piece e of a lane
    // sits at piece (e ^ n32') of its row to keep the banks apart.  One 32-row block at a time.
    constexpr int kBlkBytes = 32 * 512;                         // one block of O: 32 rows x 128 fp32
    constexpr int kLdsTotal = kLdsUsed;
    constexpr int kMlBytes = WR * 64 * 8;                       // (m, l) per lane of the parked blocks
    static_assert(KG == 1 || WR * kBlkBytes + kMlBytes <= kLdsTotal, "key-group merge staging must fit in LDS");
    if (KG > 1) {
        float *ml_park = reinterpret_cast<float *>(lds + WR * kBlkBytes);
        unsigned char *blk = lds + wave * kBlkBytes + lane * 256;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
#pragma unroll
            for (int g = 1; g < KG; ++g) {
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // ring, query fragments or the previous staging are free
                if (kg == g && rb < nrb_live) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        f32x4 o = {oacc[rb][0][e], oacc[rb][1][e], oacc[rb][2][e], oacc[rb][3][e]};
                        *reinterpret_cast<f32x4 *>(blk + ((e ^ (lane & 15)) << 4)) = o;
                    }
                    *reinterpret_cast<f32x2 *>(ml_park + (wave * 64 + lane) * 2) = f32x2{m_run[rb], l_run[rb]};
                }
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                if (kg == 0 && rb < nrb_live) {
                    const f32x2 ml_o = *reinterpret_cast<const f32x2 *>(ml_park + (wave * 64 + lane) * 2);
                    const float m_all = fmaxf(m_run[rb], ml_o[0]);
                    const float a0 = fast_exp2(m_run[rb] - m_all), ag = fast_exp2(ml_o[0] - m_all);
                    l_run[rb] = fmaf(ag, ml_o[1], l_run[rb] * a0);
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const f32x4 o = *reinterpret_cast<const f32x4 *>(blk + ((e ^ (lane & 15)) << 4));
#pragma unroll
                        for (int cb = 0; cb < 4; ++cb) oacc[rb][cb][e] = fmaf(ag, o[cb], oacc[rb][cb][e] * a0);
                    }
                    m_run[rb] = m_all;
                }
            }
        }
    }

    // ---- write the partial: (m, l) and unnormalised O for every live row ----------------------
    // O goes through LDS (free now) so that the stores cover whole 512-byte rows; a wavefront of
    // key group 0 stages one 32-row block (16 KiB) at a time.  When LDS is smaller than one block
    // per wavefront, the wavefronts take turns in groups of kSlots.
    const int n_part = p.n_split + 1;
    const int64_t part = ((int64_t)h * n_part + split) * p.n_rows_pad;
    constexpr int kSlots = kLdsTotal / kBlkBytes < WR ? kLdsTotal / kBlkBytes : WR;
    constexpr int kGroups = (WR + kSlots - 1) / kSlots;
#pragma unroll
    for (int grp = 0; grp < kGroups; ++grp) {
        if (WR * KG > 1) asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");   // LDS (or the previous group's staging) is free
        if (kg != 0 || wave / kSlots != grp) continue;
        unsigned char *region = lds + (wave % kSlots) * kBlkBytes;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            if (rb < nrb_live) {
                const int row_base = tile_row0 + (rb * WR + wave) * 32;
                const float l_tot = swap32_sum(l_run[rb]);
                if (row_base + n32 < p.n_rows && hh == 0) {
                    f32x2 ml = {m_run[rb] - m_shift, l_tot};
                    *reinterpret_cast<f32x2 *>(p.ws_ml + (part + row_base + n32) * 2) = ml;
                }
                // element e of oacc[rb][cb] is output column 32*cb + 4*hh + 8*(e/4) + e%4: four
                // consecutive elements make 16-byte piece 8*cb + 2*(e/4) + hh of row n32
#pragma unroll
                for (int cb = 0; cb < 4; ++cb)
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        f32x4 o = {oacc[rb][cb][4 * i], oacc[rb][cb][4 * i + 1], oacc[rb][cb][4 * i + 2], oacc[rb][cb][4 * i + 3]};
                        const int m = 8 * cb + 2 * i + hh;
                        *reinterpret_cast<f32x4 *>(region + n32 * 512 + ((m ^ n32) << 4)) = o;
                    }
                store_rows_from_lds<32>(region, p.n_rows - row_base, p.ws_o + (part + row_base) * kHeadDim, lane);
            }
        }
    }
}

template <int NRB, int WR, int KG, int NS, int OCC, bool QLDS, bool HALF = false>
hipError_t launch_one(const VerifyParams &p, hipStream_t stream)
{
    constexpr int kRows = 32 * NRB * WR;
    constexpr int lds_bytes = KG * NS * kStageBytes + (QLDS ? kRows * kQRowBytes : 0) + 16;   // + the note of the fp16 pass
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    static_assert(64 * WR * KG <= 1024, "workgroup size");
    if (p.rows_per_wg > kRows || p.rows_per_wg % 32 != 0) return hipErrorInvalidValue;
    static std::atomic<uint64_t> lds_allowed{0};
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(verify_wide_kernel<NRB, WR, KG, NS, OCC, QLDS, HALF>), lds_bytes, lds_allowed);
        if (e != hipSuccess) return e;
    }
    dim3 grid(p.n_split + 1, p.n_kv_heads, (p.n_rows + p.rows_per_wg - 1) / p.rows_per_wg);
    hipLaunchKernelGGL((verify_wide_kernel<NRB, WR, KG, NS, OCC, QLDS, HALF>), grid, dim3(64 * WR * KG), lds_bytes, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_verify_wide(const VerifyParams &p, int kernel_id, hipStream_t stream)
{
    switch (kernel_id) {
        case kWide_1x1: return launch_one<1, 1, 1, 3, 2, false>(p, stream);
        case kWide_1x1b: return launch_one<1, 1, 1, 4, 2, false>(p, stream);
        case kWide_1x2: return launch_one<1, 2, 1, 4, 2, false>(p, stream);
        case kWide_1x2k4: return launch_one<1, 2, 4, 2, 2, false>(p, stream);
        case kWide_1x4: return launch_one<1, 4, 1, 4, 2, false>(p, stream);
        case kWide_1x4k3: return launch_one<1, 4, 3, 2, 3, true>(p, stream);
        case kWide_2x4: return launch_one<2, 4, 1, 6, 1, false>(p, stream);
        case kWide_1x8: return launch_one<1, 8, 1, 6, 2, false>(p, stream);
        case kWide_1x10: return launch_one<1, 10, 1, 4, 3, true>(p, stream);
        case kWide_1x2h: return launch_one<1, 2, 1, 4, 2, false, true>(p, stream);
        case kWide_1x4h: return launch_one<1, 4, 1, 4, 2, false, true>(p, stream);
        case kWide_1x4k2h: return launch_one<1, 4, 2, 4, 2, false, true>(p, stream);
        case kWide_1x8h: return launch_one<1, 8, 1, 6, 2, false, true>(p, stream);
        case kWide_1x10h: return launch_one<1, 10, 1, 4, 3, true, true>(p, stream);
        case kWide_1x12h: return launch_one<1, 12, 1, 3, 3, true, true>(p, stream);
        case kWide_1x12: return launch_one<1, 12, 1, 3, 3, true>(p, stream);
        case kWide_2x2: return launch_one<2, 2, 1, 4, 1, false>(p, stream);
        case kWide_2x2k2: return launch_one<2, 2, 2, 4, 1, false>(p, stream);
        case kWide_2x2k2b: return launch_one<2, 2, 2, 3, 1, false>(p, stream);
        case kWide_1x8h4: return launch_one<1, 8, 1, 4, 2, false, true>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ts
