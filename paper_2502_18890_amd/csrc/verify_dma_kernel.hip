// Tree-masked verification attention over the full KV cache (Alg. 1 "Parallel Verification",
// App. E of the TokenSwift paper), split along the cache, for gfx950 -- variant whose K/V
// tiles go from HBM straight into LDS (buffer_load ... lds), several tiles ahead of compute.
//
// This is the kernel for at most 32 query rows per KV head (MHA, narrow trees), where the pass
// is purely HBM-bound.  One workgroup = one KV head x one contiguous range of cached tokens
// (last split index = the tree tokens with the ancestor mask); S^T = K.Q^T and O^T += V^T.P^T
// on v_mfma_f32_16x16x32_bf16 with keys on the M axis, so that all logits a lane owns belong
// to one query row; online softmax in fp32 (exp2 domain), P as bf16 hi + lo.
// A tile is 32 keys: 8 KiB of K and 8 KiB of V, unpadded.  Each wavefront load
// instruction moves four whole 256-byte rows (64 lanes x 16 B) into 1 KiB of LDS without
// touching a VGPR, so the bytes in flight are bounded by LDS (NS stages per workgroup), not
// by registers; the pass is HBM-bound and wants as many bytes in flight as it can get.
// Bank conflicts are avoided by permuting the 16-byte pieces inside each row on the way in
// (the lane that fills LDS piece `pos` of row R fetches global piece pos ^ f(R)), not by
// padding:
//   K rows: f(R) = R mod 16       -> the 16 rows an MFMA A-operand read touches land on 16
//                                    different bank groups;
//   V rows: f(R) = 8*((R/4) mod 2) -> the four rows a 64-bit V read touches (4 apart) alternate
//                                    between the two 128-byte halves of the banks.
// Rows past the end of the range are cut off by the buffer descriptor's byte count (the load
// returns zeros and moves no data); the ring is cleared once at start so that a stage never
// holds anything but finite values (a masked key contributes 0 * V).
#include <type_traits>

#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

typedef __attribute__((address_space(3))) void *lds_void_ptr;

constexpr int kTileKeys = 32;
constexpr int kStageBytes = kTileKeys * 512;   // K half then V half
constexpr int kVHalf = kTileKeys * 256;
constexpr int kQRowBytes = 272;                // padded query rows (QLDS)
constexpr float kRescaleSlack = 8.0f;          // log2 units

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// NRB: 16-row blocks per wavefront; WR: wavefronts per workgroup (along the query rows);
// NS: LDS stages (NS-1 tiles in flight while one is consumed); OCC: wavefronts per SIMD the
// register budget is cut for; QLDS: query fragments live in LDS instead of registers.
template <int NRB, int WR, int NS, int OCC, bool QLDS>
__global__ void __launch_bounds__(64 * WR) __attribute__((amdgpu_waves_per_eu(OCC, OCC)))
verify_dma_kernel(const VerifyParams p)
{
    constexpr int NT = 64 * WR;
    constexpr int LPW = 16 / WR;   // load instructions per wavefront per tile (16 x 1 KiB = one tile)
    static_assert(16 % WR == 0 && NS >= 2, "bad shape");
    static_assert((NS - 2) * LPW <= 63, "too many loads in flight for vmcnt");
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: selects which blocks this wavefront loads
    const int j = lane & 15;
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

    // ---- clear the ring --------------------------------------------------------------------
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int off = tid * 16; off < NS * kStageBytes; off += NT * 16) *reinterpret_cast<u32x4 *>(lds + off) = z;
    }
    // the cleared ring is complete before any load may write into it (LDS traffic only: no
    // need to wait for global memory here)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");

    // ---- query fragments (MFMA B operand): loads issued now, awaited after the prefetch is out --
    const int row0 = blockIdx.z * (16 * NRB * WR) + wave * NRB * 16;
    unsigned char *qlds = lds + NS * kStageBytes + (wave * NRB * 16) * kQRowBytes;
    u32x4 qraw[NRB][4];
    uint64_t amask[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int row = row0 + rb * 16 + j;
        const bool live = row < p.n_rows;
        const int node = live ? row / p.group : 0;
        const int jj = live ? row % p.group : 0;
        const uint16_t *qrow = p.q + ((int64_t)node * p.n_q_heads + h * p.group + jj) * kHeadDim;
        amask[rb] = live ? p.anc[node][0] : 0ull;   // at most 32 rows here, so at most 32 tree nodes
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (live) raw = *reinterpret_cast<const u32x4 *>(qrow + s * 32 + quad * 8);
            qraw[rb][s] = raw;
        }
    }

    float m_run[NRB], l_run[NRB];
    f32x4 oacc[NRB][2][4];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        m_run[rb] = kNegBig;
        l_run[rb] = 0.f;
#pragma unroll
        for (int dg = 0; dg < 2; ++dg)
#pragma unroll
            for (int i = 0; i < 4; ++i) oacc[rb][dg][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- HBM -> LDS -------------------------------------------------------------------------
    // Load instruction ii (0..15) of a tile fills LDS block ii: K rows 4ii..4ii+3 for ii < 8,
    // V rows 4(ii-8).. for ii >= 8.  This wavefront issues ii = wave*LPW .. wave*LPW+LPW-1.
    uint32_t goff[LPW];
#pragma unroll
    for (int i = 0; i < LPW; ++i) {
        const int ii = wave * LPW + i;
        const int R = 4 * (ii & 7) + quad;                       // row of the tile this lane fetches from
        const int f = (ii >= 8) ? (((R >> 2) & 1) << 3) : (R & 15);
        goff[i] = (uint32_t)(R * tstride * 2 + ((j ^ f) << 4));
    }
    // Tiles are issued and consumed strictly in order, so both sides keep running cursors (a few
    // scalar additions per tile) instead of recomputing addresses from the tile number.
    constexpr uint32_t kRingBytes = NS * kStageBytes;
    const int64_t tile_elems = (int64_t)kTileKeys * tstride;     // elements between consecutive tiles
    const uint16_t *kfill = kbase + t_begin * tstride;
    const uint16_t *vfill = vbase + t_begin * tstride;
    // bytes from the first row of the next tile to fill up to the end of the last valid row (<= 0: none)
    int64_t fill_rem = (t_end - t_begin - 1) * tstride * 2 + 256;
    uint32_t fill_stage = 0;
    auto issue_tile = [&]() {
        const uint32_t nrec = fill_rem <= 0 ? 0u : (fill_rem > 0xffffffffLL ? 0xffffffffu : (uint32_t)fill_rem);
        const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(kfill), 0, nrec, 0x00020000);
        const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t *>(vfill), 0, nrec, 0x00020000);
        unsigned char *stage = lds + fill_stage;
#pragma unroll
        for (int i = 0; i < LPW; ++i) {
            const int ii = wave * LPW + i;                       // wave-uniform
            const uint32_t go = goff[i];   // (a local copy: the builtin rejects an element of a template-sized array on the host pass)
            if (ii < 8)
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rk, (lds_void_ptr)(stage + ii * 1024), 16, go, 0, 0, kCachePolicyStream);
            else
                __builtin_amdgcn_raw_ptr_buffer_load_lds(rv, (lds_void_ptr)(stage + kVHalf + (ii - 8) * 1024), 16, go, 0, 0, kCachePolicyStream);
        }
        kfill += tile_elems;     // past the range the descriptor covers 0 bytes, so the base is never dereferenced
        vfill += tile_elems;
        fill_rem -= tile_elems * 2;
        fill_stage += kStageBytes;
        if (fill_stage >= kRingBytes) fill_stage = 0;
    };

    // per-lane LDS read offsets inside a stage
    int koff[4];   // K: row j of a 16-row block, piece (4s + quad) ^ j
#pragma unroll
    for (int s = 0; s < 4; ++s) koff[s] = j * 256 + ((((s << 2) | quad) ^ j) << 4);
    int voffl[2];  // V: row quad*4 of a 16-row block, columns 4j..4j+3 of 64-column half dg
#pragma unroll
    for (int dg = 0; dg < 2; ++dg)
        voffl[dg] = kVHalf + quad * 1024 + ((((dg << 3) | (j >> 1)) ^ ((quad & 1) << 3)) << 4) + ((j & 1) << 3);

    const int n_tiles = (int)((t_end - t_begin + kTileKeys - 1) / kTileKeys);
#pragma unroll
    for (int s = 0; s < NS - 1; ++s) issue_tile();   // tiles past the range load nothing but still count

    // Now wait for the query and mask loads (older than every tile load, so the tile loads stay
    // in flight) -- here, not at their first use inside the main loop, where the wait would be
    // for everything issued before it, i.e. for the whole prefetched ring.
    bf16x8 qf[QLDS ? 1 : NRB][4];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        asm volatile("" ::"v"(amask[rb]));
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            asm volatile("" ::"v"(qraw[rb][s]));
            if (QLDS)   // each wavefront later reads back only what it wrote itself
                *reinterpret_cast<u32x4 *>(qlds + (rb * 16 + j) * kQRowBytes + (s * 32 + quad * 8) * 2) = qraw[rb][s];
            else
                qf[rb][s] = __builtin_bit_cast(bf16x8, qraw[rb][s]);
        }
    }

    // Tile sums for the chunk scores (see process_tile).  The store of a tile's sum waits until just
    // before the next loads are issued: vmcnt counts loads and stores alike, in order, so a store younger
    // than the loads a step waits for would put its own latency on that wait.
    const bool scoring = p.tile_sums != nullptr && wave == 0 && blockIdx.z == 0 && !is_tree;   // wavefront-uniform
    float score_parked = 0.f;
    int64_t score_parked_tile = -1;
    auto score_flush = [&]() {
        if (scoring && score_parked_tile >= 0) {
            if (lane == 0) p.tile_sums[(int64_t)h * p.tile_sums_stride + score_parked_tile] = score_parked;
            score_parked_tile = -1;
        }
    };

    // One 32-key tile against all of this wavefront's rows.  RAGGED tiles (the last one of a
    // range, every tile of the tree split) mask keys; full tiles carry no masking code at all.
    // The body is laid out as three straight-line blocks so that the scheduler can overlap
    // matrix and vector work: (1) S^T MFMAs with the V^T operand regrouping, (2) row maxima of
    // all row blocks and one ballot (rescaling is a rare side branch), (3) exp/pack of row
    // block rb+1 against the PV MFMAs of row block rb.
    auto process_tile = [&](auto ragged_tag, const unsigned char *stage, int64_t t0) {
        constexpr bool RAGGED = decltype(ragged_tag)::value;

        // ---- (1) S^T = K . Q^T for the 32 keys; V^T operands ---------------------------------
        f32x4 sacc[NRB][2];
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            sacc[rb][0] = f32x4{0.f, 0.f, 0.f, 0.f};
            sacc[rb][1] = f32x4{0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(stage + kb * 4096 + koff[s]);
#pragma unroll
                for (int rb = 0; rb < NRB; ++rb) {
                    const bf16x8 b = QLDS ? *reinterpret_cast<const bf16x8 *>(
                                                qlds + (rb * 16 + j) * kQRowBytes + (s * 32 + quad * 8) * 2)
                                          : qf[QLDS ? 0 : rb][s];
                    sacc[rb][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, sacc[rb][kb], 0, 0, 0);
                }
            }
        }
        // Chunk scores ride along: the rows of the first tree node (rows 0..group-1, in wavefront 0) hold
        // exactly the raw logits q.k that Eq. 2 sums; their sum over the tile's valid keys is parked
        // until the next tile's loads are about to be issued (see score_flush), and the merge kernel
        // turns tiles into chunks.
        // (This lane's own eight logits are added here, while they are at hand; the cross-lane part of the sum waits
        // until the second product's matrix instructions have been issued and runs in their shadow.)
        const bool score_this = scoring && t0 < t_end;
        float ssum = 0.f;
        if (score_this) {
            const uint32_t ok = RAGGED ? (uint32_t)((t_end - t0 >= 32 ? 0xffffffffull : ((1ull << (t_end - t0)) - 1ull)) >> (quad * 4)) : 0xffffffffu;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float v = sacc[0][e >> 2][e & 3];
                ssum += (!RAGGED || ((ok >> ((e >> 2) * 16 + (e & 3))) & 1u)) ? v : 0.f;
            }
        }
        // 8 keys x 4 consecutive columns per read, regrouped into one column x 8 keys per operand
        bf16x8 av[2][4];
#pragma unroll
        for (int dg = 0; dg < 2; ++dg) {
            u32x2 vr[8];
#pragma unroll
            for (int e = 0; e < 8; ++e)
                vr[e] = *reinterpret_cast<const u32x2 *>(stage + ((e >> 2) * 16 + (e & 3)) * 256 + voffl[dg]);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                u32x4 a;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t x = vr[2 * w][i >> 1], y = vr[2 * w + 1][i >> 1];
                    a[w] = (i & 1) ? __builtin_amdgcn_perm(y, x, 0x07060302u) : __builtin_amdgcn_perm(y, x, 0x05040100u);
                }
                av[dg][i] = __builtin_bit_cast(bf16x8, a);
            }
        }

        // ---- (2) row maxima (raw logits; scale > 0 commutes with max) --------------------------
        // This lane owns keys kb*16 + quad*4 + v (e = kb*4 + v) of query row j.
        // m_run is a reference point, not necessarily the exact running maximum: the accumulators
        // are rescaled only when a tile's maximum exceeds it by more than kRescaleSlack, so the
        // weights stay <= 2^kRescaleSlack and the (rare) rescale leaves the common path.
        float m_tile[NRB];
        bool moved = false;
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            if (RAGGED) {
                // bit b of vm: key quad*4 + b of this tile may be attended by row j
                const uint64_t tile_ok = is_tree ? (amask[rb] >> t0)
                                                 : (t_end - t0 >= 64 ? ~0ull : ((1ull << (t_end - t0)) - 1ull));
                const uint32_t vm = (uint32_t)(tile_ok >> (quad * 4));
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (!((vm >> ((e >> 2) * 16 + (e & 3))) & 1u)) sacc[rb][e >> 2][e & 3] = -INFINITY;
            }
            const f32x4 s0 = sacc[rb][0], s1 = sacc[rb][1];
            float mloc = fmaxf(fmaxf(fmaxf(s0[0], s0[1]), fmaxf(s0[2], s0[3])), fmaxf(fmaxf(s1[0], s1[1]), fmaxf(s1[2], s1[3])));
            m_tile[rb] = xrow_max(mloc) * p.scale_log2;
            moved |= (m_tile[rb] > m_run[rb] + kRescaleSlack);
        }
        if (__builtin_amdgcn_ballot_w64(moved) != 0ull) {   // some row of this wavefront outgrew its reference
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) {
                const float m_new = fmaxf(m_run[rb], m_tile[rb]);
                const float alpha = fast_exp2(m_run[rb] - m_new);
                l_run[rb] *= alpha;
#pragma unroll
                for (int dg = 0; dg < 2; ++dg)
#pragma unroll
                    for (int i = 0; i < 4; ++i) oacc[rb][dg][i] *= alpha;
                m_run[rb] = m_new;
            }
        }

        // ---- (3) P = exp2(scale*s - m), split hi + lo (both bf16), O^T += V^T . P^T -------------
        // Software-pipelined over the row blocks: the vector work that makes P of block rb+1 sits
        // in the same scheduling region as the matrix work that consumes P of block rb.
        auto make_p = [&](int rb, bf16x8 &p_hi, bf16x8 &p_lo) {
            float pe[8], psum = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                pe[e] = fast_exp2(fmaf(sacc[rb][e >> 2][e & 3], p.scale_log2, -m_run[rb]));
                psum += pe[e];
            }
            l_run[rb] += psum;
            u32x4 hi, lo;   // the product keeps ~16 bits of each weight
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const uint32_t hw = pack_bf16(pe[2 * w], pe[2 * w + 1]);
                hi[w] = hw;
                lo[w] = pack_bf16(pe[2 * w] - bf16lo_to_f32(hw), pe[2 * w + 1] - bf16hi_to_f32(hw));
            }
            p_hi = __builtin_bit_cast(bf16x8, hi);
            p_lo = __builtin_bit_cast(bf16x8, lo);
        };
        bf16x8 p_hi[2], p_lo[2];
        make_p(0, p_hi[0], p_lo[0]);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
            if (rb + 1 < NRB) make_p(rb + 1, p_hi[(rb + 1) & 1], p_lo[(rb + 1) & 1]);
#pragma unroll
            for (int dg = 0; dg < 2; ++dg)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    oacc[rb][dg][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[dg][i], p_hi[rb & 1], oacc[rb][dg][i], 0, 0, 0);
#pragma unroll
            for (int dg = 0; dg < 2; ++dg)
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    oacc[rb][dg][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[dg][i], p_lo[rb & 1], oacc[rb][dg][i], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (score_this) {
            ssum = xrow_sum(ssum);                                   // the four lanes that share row j
            score_parked = row16_sum(j < p.group ? ssum : 0.f);     // the group's heads
            score_parked_tile = t0 >> 5;
        }
    };

    // full tiles first, then (cache ranges) at most one ragged tile; the tree split is all ragged
    uint32_t use_stage = 0;          // stage of the tile being consumed
    int64_t t0_cur = t_begin;        // its first token
    auto step = [&](auto ragged_tag) {
        // this wavefront's pieces of the next tile have landed (a parked tile sum, stored just before
        // the newest tile's loads were issued, is one more operation allowed to be outstanding)
        if (scoring) wait_vmcnt<(NS - 2) * LPW + (NS > 2 ? 1 : 0)>();
        else wait_vmcnt<(NS - 2) * LPW>();
        // ... and everyone's; all are done with the previous tile.  A bare s_barrier: __syncthreads() would add a
        // fence that waits for every outstanding load, i.e. for the whole prefetched ring.
        if (WR > 1) asm volatile("s_barrier" ::: "memory");
        score_flush();
        issue_tile();                                 // refill the stage that the previous tile occupied
        process_tile(ragged_tag, lds + use_stage, t0_cur);
        use_stage += kStageBytes;
        if (use_stage >= kRingBytes) use_stage = 0;
        t0_cur += kTileKeys;
    };
    const int n_full = is_tree ? 0 : (int)((t_end - t_begin) / kTileKeys);
    for (int it = 0; it < n_full; ++it) step(std::false_type{});
    for (int it = n_full; it < n_tiles; ++it) step(std::true_type{});
    score_flush();
    wait_vmcnt<0>();   // drain the loads issued past the range before the workgroup's LDS is released

    // ---- write the partial: (m, l) and unnormalised O for every live row ----------------------
    // O goes through LDS (the ring is free now) so that the stores cover whole 512-byte rows.
    if (WR > 1) asm volatile("s_barrier" ::: "memory");   // every wavefront is done with the ring, no load still targets it
    unsigned char *region = lds + wave * (NRB * 16 * 512);
    static_assert(WR * NRB * 16 * 512 <= NS * kStageBytes, "write-back staging must fit in the ring");
    const int n_part = p.n_split + 1;
    const int64_t part = ((int64_t)h * n_part + split) * p.n_rows_pad;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int row = row0 + rb * 16 + j;
        const float l_tot = xrow_sum(l_run[rb]);
        if (row < p.n_rows && quad == 0) {
            f32x2 ml = {m_run[rb], l_tot};
            *reinterpret_cast<f32x2 *>(p.ws_ml + (part + row) * 2) = ml;
        }
        // this lane holds columns dg*64 + quad*16 + 4v + i of row j: 16-byte piece dg*16 + quad*4 + v
        unsigned char *blk = region + rb * (16 * 512);
#pragma unroll
        for (int dg = 0; dg < 2; ++dg)
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                f32x4 o = {oacc[rb][dg][0][v], oacc[rb][dg][1][v], oacc[rb][dg][2][v], oacc[rb][dg][3][v]};
                *reinterpret_cast<f32x4 *>(blk + j * 512 + (((dg * 16 + quad * 4 + v) ^ j) << 4)) = o;
            }
        const int row_base = row0 + rb * 16;
        if (row_base < p.n_rows)
            store_rows_from_lds<16>(blk, p.n_rows - row_base, p.ws_o + (part + row_base) * kHeadDim, lane);
    }
}

template <int NRB, int WR, int NS, int OCC, bool QLDS>
hipError_t launch_one(const VerifyParams &p, hipStream_t stream)
{
    constexpr int kRows = 16 * NRB * WR;
    constexpr int lds_bytes = NS * kStageBytes + (QLDS ? kRows * kQRowBytes : 0);
    static_assert(lds_bytes <= 160 * 1024, "LDS budget");
    static std::atomic<uint64_t> lds_allowed{0};
    if (lds_bytes > 64 * 1024) {
        const hipError_t e = allow_dynamic_lds(reinterpret_cast<const void *>(verify_dma_kernel<NRB, WR, NS, OCC, QLDS>), lds_bytes, lds_allowed);
        if (e != hipSuccess) return e;
    }
    dim3 grid(p.n_split + 1, p.n_kv_heads, (p.n_rows + kRows - 1) / kRows);
    hipLaunchKernelGGL((verify_dma_kernel<NRB, WR, NS, OCC, QLDS>), grid, dim3(64 * WR), lds_bytes, stream, p);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_verify_narrow(const VerifyParams &p, int kernel_id, hipStream_t stream)
{
    switch (kernel_id) {
        case kNarrow_16: return launch_one<1, 1, 2, 2, false>(p, stream);
        case kNarrow_32: return launch_one<1, 2, 2, 2, false>(p, stream);   // 4 workgroups per CU
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ts
