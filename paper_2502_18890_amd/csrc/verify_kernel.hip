// Tree-masked verification attention over the full KV cache (Alg. 1 "Parallel Verification",
// App. E of the TokenSwift paper), split along the cache ("split-K"), for gfx950.
//
// One workgroup = one KV head x one contiguous range of cached tokens (or, for the last
// split index, the tree tokens themselves with the ancestor mask).  All R = g*T query rows
// that share this KV head are processed against every K/V tile the workgroup streams, so
// each cached byte is read from HBM exactly once per call:
//
//   S^T[key][row] = K_tile . Q^T          v_mfma_f32_16x16x32_bf16, keys on the M axis
//   online softmax over keys, per row      fp32 VALU, exp2 domain
//   O^T[d][row]  += V_tile^T . P^T         same MFMA, P split into bf16 hi + lo parts
//
// Keys sit on the MFMA M axis so that the 4 (per 16 keys) logits a lane owns all belong to
// one query row: the running max/sum stay per-lane state and the rescale of the O^T
// accumulators is a per-lane scalar multiply.  K/V tiles go HBM -> registers (128-bit
// loads, next tile in flight during compute) -> LDS (padded rows) -> MFMA operands; the
// WR wavefronts of a workgroup each own 16*NRB query rows and share the LDS tile.
// The workgroup writes (m, l, unnormalised O) per row; combine_kernel merges the splits.
#include "ts_device.hpp"
#include "ts_internal.hpp"

namespace ts {

namespace {

constexpr int kKRowBytes = 272;  // 256 B of keys + 16 B pad: 16 rows x 16 B reads hit distinct banks
constexpr int kVRowBytes = 288;  // 256 B of values + 32 B pad: rows 4 apart are 32 banks apart

template <int BK, int NSLOT>
struct VerifyLds {
    static constexpr int kSlotBytes = BK * (kKRowBytes + kVRowBytes);
    static constexpr int kBytes = NSLOT * kSlotBytes;
};

// NRB: 16-row blocks per wavefront; WR: wavefronts per workgroup (all along the row axis);
// BK: keys per tile (multiple of 32); OCC: wavefronts per SIMD the register budget is cut for;
// QLDS: keep the query fragments in LDS instead of registers (for many rows per wavefront).
// blockIdx.z selects a tile of 16*NRB*WR query rows when one workgroup cannot hold them all
// (the cache is then streamed once per row tile).
template <int NRB, int WR, int BK, int OCC, bool QLDS>
__global__ void __launch_bounds__(64 * WR) __attribute__((amdgpu_waves_per_eu(OCC, OCC)))
verify_kernel(const VerifyParams p)
{
    constexpr int NT = 64 * WR;
    constexpr int NSLOT = (WR > 1) ? 2 : 1;
    constexpr int CHUNKS = BK * 16;           // 16-byte pieces of the K tile (same for V)
    static_assert(CHUNKS % NT == 0, "tile must divide evenly over the threads");
    constexpr int LPT = 2 * CHUNKS / NT;      // 128-bit loads per thread per tile (K then V)
    extern __shared__ __attribute__((aligned(16))) unsigned char lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int j = lane & 15;     // MFMA column: query row inside a 16-row block / key row for A
    const int quad = lane >> 4;  // MFMA k-group
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

    // ---- query fragments (MFMA B operand), resident for the whole kernel -------------------
    // in registers, or (QLDS) in an LDS area behind the tile slots, one padded row per query row
    const int row0 = blockIdx.z * (16 * NRB * WR) + wave * NRB * 16;
    unsigned char *qlds = lds + VerifyLds<BK, NSLOT>::kBytes + (wave * NRB * 16) * kKRowBytes;
    bf16x8 qf[QLDS ? 1 : NRB][4];
    uint64_t amask[NRB];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int row = row0 + rb * 16 + j;
        const bool live = row < p.n_rows;
        const int node = live ? row / p.group : 0;
        const int jj = live ? row % p.group : 0;
        const uint16_t *qrow = p.q + ((int64_t)node * p.n_q_heads + h * p.group + jj) * kHeadDim;
        amask[rb] = live ? p.anc[node] : 0ull;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            u32x4 raw = {0u, 0u, 0u, 0u};
            if (live) raw = *reinterpret_cast<const u32x4 *>(qrow + s * 32 + quad * 8);
            if (QLDS)
                *reinterpret_cast<u32x4 *>(qlds + (rb * 16 + j) * kKRowBytes + (s * 32 + quad * 8) * 2) = raw;
            else
                qf[rb][s] = __builtin_bit_cast(bf16x8, raw);
        }
    }
    // (QLDS: each wavefront reads back only what it wrote itself; LDS ops of a wavefront stay in order)

    // ---- running softmax state and output accumulators ------------------------------------
    float m_run[NRB], l_run[NRB];
    f32x4 oacc[NRB][2][4];  // [row block][64-column half][column i within a group of 4]
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        m_run[rb] = kNegBig;
        l_run[rb] = 0.f;
#pragma unroll
        for (int dg = 0; dg < 2; ++dg)
#pragma unroll
            for (int i = 0; i < 4; ++i) oacc[rb][dg][i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    // ---- HBM -> register staging ----------------------------------------------------------
    // Buffer loads with a per-tile resource descriptor: the descriptor's byte count ends at
    // the last valid row of the range, so pieces of rows past it come back as zeros (V must
    // be finite for masked keys) without any per-load branch, and a lane needs only one
    // 32-bit offset per piece, the same for every tile.
    u32x4 stage[LPT];
    uint32_t voff[LPT / 2];
#pragma unroll
    for (int i = 0; i < LPT / 2; ++i) {
        const int cc = i * NT + tid;
        voff[i] = (uint32_t)((cc >> 4) * tstride * 2 + (cc & 15) * 16);
    }
    auto issue_loads = [&](int64_t t0) {
        const int64_t span = (t_end - t0 - 1) * tstride * 2 + 256;   // bytes up to the end of the last valid row
        const uint32_t nrec = span > 0xffffffffLL ? 0xffffffffu : (uint32_t)span;
        const __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(kbase + t0 * tstride), 0, nrec, 0x00020000);
        const __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(vbase + t0 * tstride), 0, nrec, 0x00020000);
#pragma unroll
        for (int i = 0; i < LPT / 2; ++i)
            stage[i] = __builtin_amdgcn_raw_buffer_load_b128(rk, voff[i], 0, 0);
#pragma unroll
        for (int i = 0; i < LPT / 2; ++i)
            stage[LPT / 2 + i] = __builtin_amdgcn_raw_buffer_load_b128(rv, voff[i], 0, 0);
    };
    auto store_tile = [&](unsigned char *slot) {
#pragma unroll
        for (int i = 0; i < LPT; ++i) {
            const bool is_v = (i * NT >= CHUNKS);
            const int cc = i * NT + tid - (is_v ? CHUNKS : 0);
            const int r = cc >> 4, c16 = cc & 15;
            unsigned char *dst = is_v ? slot + BK * kKRowBytes + r * kVRowBytes + c16 * 16
                                      : slot + r * kKRowBytes + c16 * 16;
            *reinterpret_cast<u32x4 *>(dst) = stage[i];
        }
    };

    const int64_t n_tiles = (t_end - t_begin + BK - 1) / BK;
    if (n_tiles > 0) issue_loads(t_begin);

    for (int64_t it = 0; it < n_tiles; ++it) {
        const int64_t t0 = t_begin + it * BK;
        unsigned char *slot = lds + (NSLOT > 1 ? (it & 1) * VerifyLds<BK, NSLOT>::kSlotBytes : 0);
        store_tile(slot);
        if (it + 1 < n_tiles) issue_loads(t0 + BK);
        if (WR > 1)
            __syncthreads();
        else
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // one wavefront: LDS ops stay in program order

        const unsigned char *ldsK = slot;
        const unsigned char *ldsV = slot + BK * kKRowBytes;
        const bool ragged = is_tree || (t0 + BK > t_end);

#pragma unroll
        for (int sb = 0; sb < BK / 32; ++sb) {
            // ---- S^T = K . Q^T for 32 keys --------------------------------------------
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
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(
                        ldsK + (sb * 32 + kb * 16 + j) * kKRowBytes + (s * 32 + quad * 8) * 2);
#pragma unroll
                    for (int rb = 0; rb < NRB; ++rb) {
                        const bf16x8 b = QLDS ? *reinterpret_cast<const bf16x8 *>(
                                                    qlds + (rb * 16 + j) * kKRowBytes + (s * 32 + quad * 8) * 2)
                                              : qf[QLDS ? 0 : rb][s];
                        sacc[rb][kb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, sacc[rb][kb], 0, 0, 0);
                    }
                }
            }

            // ---- V^T operands for the 32 keys --------------------------------------------
            // The lane reads, for each of its 8 keys, the 4 consecutive columns 4j..4j+3 of a
            // 64-column half and regroups them into 4 operands (one column, 8 keys each).
            bf16x8 av[2][4];
#pragma unroll
            for (int dg = 0; dg < 2; ++dg) {
                u32x2 vr[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int key = sb * 32 + (e >> 2) * 16 + quad * 4 + (e & 3);
                    vr[e] = *reinterpret_cast<const u32x2 *>(ldsV + key * kVRowBytes + dg * 128 + j * 8);
                }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    u32x4 a;
#pragma unroll
                    for (int w = 0; w < 4; ++w) {
                        const uint32_t x = vr[2 * w][i >> 1], y = vr[2 * w + 1][i >> 1];
                        a[w] = (i & 1) ? __builtin_amdgcn_perm(y, x, 0x07060302u)
                                       : __builtin_amdgcn_perm(y, x, 0x05040100u);
                    }
                    av[dg][i] = __builtin_bit_cast(bf16x8, a);
                }
            }

            // ---- per 16-row block: online softmax, then O^T += V^T . P^T ------------------
            // This lane owns keys kb*16 + quad*4 + v (e = kb*4 + v) of query row j.
#pragma unroll
            for (int rb = 0; rb < NRB; ++rb) {
                float t[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) t[e] = sacc[rb][e >> 2][e & 3] * p.scale_log2;
                if (ragged) {
                    // bit b of vm: key sb*32 + quad*4 + b of this tile may be attended by row j
                    const uint64_t tile_ok = is_tree ? (amask[rb] >> t0)
                                                     : (t_end - t0 >= 64 ? ~0ull : ((1ull << (t_end - t0)) - 1ull));
                    const uint32_t vm = (uint32_t)(tile_ok >> (sb * 32 + quad * 4));
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        t[e] = ((vm >> ((e >> 2) * 16 + (e & 3))) & 1u) ? t[e] : -INFINITY;
                }
                float mloc = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])),
                                   fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
                mloc = xrow_max(mloc);
                const float m_new = fmaxf(m_run[rb], mloc);
                // rescale only when some row of this block saw a new maximum
                if (__builtin_amdgcn_ballot_w64(m_new != m_run[rb]) != 0ull) {
                    const float alpha = fast_exp2(m_run[rb] - m_new);
                    l_run[rb] *= alpha;
#pragma unroll
                    for (int dg = 0; dg < 2; ++dg)
#pragma unroll
                        for (int i = 0; i < 4; ++i) oacc[rb][dg][i] *= alpha;
                    m_run[rb] = m_new;
                }
                float pe[8], psum = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    pe[e] = fast_exp2(t[e] - m_new);
                    psum += pe[e];
                }
                l_run[rb] += psum;
                // P = hi + lo with both parts bf16: the product keeps ~16 bits of each weight
                u32x4 hi, lo;
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    const uint32_t hw = pack_bf16(pe[2 * w], pe[2 * w + 1]);
                    hi[w] = hw;
                    lo[w] = pack_bf16(pe[2 * w] - bf16lo_to_f32(hw), pe[2 * w + 1] - bf16hi_to_f32(hw));
                }
                const bf16x8 p_hi = __builtin_bit_cast(bf16x8, hi);
                const bf16x8 p_lo = __builtin_bit_cast(bf16x8, lo);
#pragma unroll
                for (int dg = 0; dg < 2; ++dg)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        oacc[rb][dg][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[dg][i], p_hi, oacc[rb][dg][i], 0, 0, 0);
#pragma unroll
                for (int dg = 0; dg < 2; ++dg)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        oacc[rb][dg][i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av[dg][i], p_lo, oacc[rb][dg][i], 0, 0, 0);
            }
        }
        // with one slot (WR == 1) the same wavefront rewrites it only after its own reads;
        // with two slots the barrier of the next iteration orders reads before the rewrite
    }

    // ---- write the partial: (m, l) and unnormalised O for every live row -------------------
    const int n_part = p.n_split + 1;
    const int64_t part = ((int64_t)h * n_part + split) * p.n_rows_pad;
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb) {
        const int row = row0 + rb * 16 + j;
        const float l_tot = xrow_sum(l_run[rb]);
        if (row < p.n_rows) {
            if (quad == 0) {
                f32x2 ml = {m_run[rb], l_tot};
                *reinterpret_cast<f32x2 *>(p.ws_ml + (part + row) * 2) = ml;
            }
            float *orow = p.ws_o + (part + row) * kHeadDim;
            // this lane holds columns dg*64 + quad*16 + 4v + i
#pragma unroll
            for (int dg = 0; dg < 2; ++dg)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    f32x4 o = {oacc[rb][dg][0][v], oacc[rb][dg][1][v], oacc[rb][dg][2][v], oacc[rb][dg][3][v]};
                    *reinterpret_cast<f32x4 *>(orow + dg * 64 + quad * 16 + 4 * v) = o;
                }
        }
    }
}

template <int NRB, int WR, int BK, int OCC, bool QLDS>
hipError_t launch_one(const VerifyParams &p, hipStream_t stream)
{
    constexpr int NSLOT = (WR > 1) ? 2 : 1;
    constexpr int kRows = 16 * NRB * WR;
    constexpr int lds_bytes = VerifyLds<BK, NSLOT>::kBytes + (QLDS ? kRows * kKRowBytes : 0);
    static bool attr_set = false;
    if (lds_bytes > 64 * 1024 && !attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(verify_kernel<NRB, WR, BK, OCC, QLDS>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    dim3 grid(p.n_split + 1, p.n_kv_heads, (p.n_rows + kRows - 1) / kRows);
    hipLaunchKernelGGL((verify_kernel<NRB, WR, BK, OCC, QLDS>), grid, dim3(64 * WR), lds_bytes, stream, p);
    return hipGetLastError();
}

}  // namespace

// Row pitch of the workspace: rows are padded to what the chosen kernel shape covers.
int verify_rows_capacity(int n_rows)
{
    if (n_rows < 1 || n_rows > 512) return 0;
    if (n_rows <= 16) return 16;
    if (n_rows <= 32) return 32;
    if (n_rows <= 64) return 64;
    if (n_rows <= 96) return 96;
    if (n_rows <= 128) return 128;
    if (n_rows <= 192) return 192;
    if (n_rows <= 256) return 256;
    if (n_rows <= 320) return 320;
    if (n_rows <= 384) return 384;
    return 512;   // two row tiles of 256
}

hipError_t launch_verify(const VerifyParams &p, hipStream_t stream)
{
    switch (verify_rows_capacity(p.n_rows)) {
        case 16: return launch_one<1, 1, 32, 2, false>(p, stream);
        case 32: return launch_one<1, 2, 32, 2, false>(p, stream);
        case 64: return launch_one<2, 2, 32, 2, false>(p, stream);
        case 96: return launch_one<3, 2, 32, 1, false>(p, stream);
        case 128: return launch_one<2, 4, 32, 2, false>(p, stream);
        case 192: return launch_one<3, 4, 32, 1, false>(p, stream);
        case 256: return launch_one<4, 4, 32, 1, false>(p, stream);
        case 320: return launch_one<5, 4, 32, 1, true>(p, stream);
        case 384: return launch_one<6, 4, 32, 1, true>(p, stream);
        case 512: return launch_one<4, 4, 32, 1, false>(p, stream);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace ts
