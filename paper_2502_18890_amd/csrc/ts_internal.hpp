// Host <-> kernel parameter blocks and launcher declarations (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <atomic>

namespace ts {

// Kernels that use more than 64 KiB of dynamic LDS must be told so once per device; `done` is the
// launcher's own bit mask of devices already served (devices >= 64 are simply asked every time).
inline hipError_t allow_dynamic_lds(const void *kernel, int bytes, std::atomic<uint64_t> &done)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev >= 0 && dev < 64 && ((done.load(std::memory_order_relaxed) >> dev) & 1ull)) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess && dev >= 0 && dev < 64) done.fetch_or(1ull << dev, std::memory_order_relaxed);
    return e;
}


// ---- tree verification (verify_dma_kernel.hip, verify_wide_kernel.hip) ----------------------
constexpr int kMaxTree = 128;
struct VerifyParams {
    const uint16_t *q;        // bf16 [n_tree][n_q_heads][128]
    const uint16_t *k;        // cache keys
    const uint16_t *v;        // cache values
    const uint16_t *k_tree;   // bf16 [n_tree][n_kv_heads][128]
    const uint16_t *v_tree;
    float *ws_o;              // [n_kv_heads][n_split+1][n_rows_pad][128]
    float *ws_ml;             // [n_kv_heads][n_split+1][n_rows_pad][2]  (max in exp2 domain, sum)
    float *tile_sums;         // nullptr, or [n_kv_heads][tile_sums_stride]: per 32-key tile of the cache, the sum over its
                              // valid keys of the raw logits q.k of the first tree node's query heads of the group
    int64_t tile_sums_stride;
    int64_t stride_head, stride_token;
    int64_t n_tokens;
    int64_t split_len;        // cached tokens per split, multiple of 32
    int n_split;              // number of cache splits (0 if the cache is empty); index n_split = tree
    int n_q_heads, n_kv_heads, group, n_tree;
    int n_rows;               // group * n_tree; row = node * group + head within the group
    int n_rows_pad;           // row pitch of the workspace
    int rows_per_wg;          // query rows one workgroup covers (grid.z = ceil(n_rows / rows_per_wg))
    float scale_log2;         // scale * log2(e)
    uint64_t anc[kMaxTree][2];   // bit u of the 128-bit anc[i] set iff tree node u is i or an ancestor of i
};

// Which kernel instantiation serves a number of query rows per KV head, and what the split
// heuristic needs to know about it.
enum VerifyKernelId {
    kNarrow_16 = 0,   // 16x16x32 MFMA kernel, 1 wavefront x 16 rows
    kNarrow_32,       // 16x16x32 MFMA kernel, 2 wavefronts x 16 rows
    // 32x32x16 MFMA kernel, <32-row blocks per wavefront> x <wavefronts along the rows>
    kWide_1x1,
    kWide_1x1b,       // deeper ring, two workgroups per CU
    kWide_1x2,
    kWide_1x2k4,      // four key groups
    kWide_1x4,
    kWide_1x4k3,      // three key groups, query fragments in LDS
    kWide_2x4,
    kWide_1x8,
    kWide_1x10,       // query fragments in LDS
    kWide_1x12,       // query fragments in LDS
    // the same shapes with the second product in fp16 wherever the values fit
    kWide_1x2h,
    kWide_1x4h,
    kWide_1x4k2h,
    kWide_1x8h,
    kWide_1x10h,
    kWide_1x12h,
    // two row blocks per wavefront (K and V^T operands read from LDS once for both), one wavefront per SIMD
    kWide_2x2,        // two workgroups of two wavefronts per CU
    kWide_2x2k2,      // two key groups
    kWide_2x2k2b,     // ... with a three-stage ring
    kWide_1x8h4,      // 1x8h with a four-stage ring (stage offsets as immediates)
    kVerifyKernelCount
};
// rows one workgroup of a kernel covers at most, and workgroups of it a CU holds (0 rows: no such kernel)
struct VerifyKernelInfo { int max_rows; int wg_per_cu; };
VerifyKernelInfo verify_kernel_info(int kernel_id);
struct VerifyShape {
    int kernel_id;
    int rows_per_wg;   // rows covered by one workgroup (multiple of 32 for the wide kernel)
    int wg_per_cu;     // workgroups of this shape one CU holds at a time
};
bool verify_shape(int n_rows, int n_kv_heads, int64_t n_tokens, int variant, VerifyShape *out);   // false if n_rows is out of range
hipError_t launch_verify_narrow(const VerifyParams &p, int kernel_id, hipStream_t stream);
hipError_t launch_verify_wide(const VerifyParams &p, int kernel_id, hipStream_t stream);

// ---- partial-KV attention (partial_kernel.hip) ---------------------------------------------
struct PartialParams {
    const uint16_t *q;        // bf16 [n_q_heads][128]
    const uint16_t *k;
    const uint16_t *v;
    const int32_t *chunk_idx; // [n_kv_heads][n_sel]
    float *ws_o;              // [n_kv_heads][n_part][group][128]
    float *ws_ml;             // [n_kv_heads][n_part][group][2]
    int64_t stride_head, stride_token;
    int64_t n_tokens;
    int n_q_heads, n_kv_heads, group;
    int n_sel, chunk_size;
    int segs_per_chunk;       // chunk_size / 8: a 16-lane row handles one 8-token segment
    int n_seg;                // n_sel * segs_per_chunk
    int n_part;               // workgroups per KV head = ceil(n_seg / 16), one partial each
    float scale_log2;
};
hipError_t launch_partial(const PartialParams &p, hipStream_t stream);

// ---- merge of split partials (combine_kernel.hip) ------------------------------------------
struct CombineParams {
    const float *ws_o;        // [n_kv_heads][n_part][row_pitch][128]
    const float *ws_ml;       // [n_kv_heads][n_part][row_pitch][2]
    float *out;               // [n_nodes][n_q_heads][128]
    float *lse;               // [n_nodes][n_q_heads] or nullptr
    int n_kv_heads, n_q_heads, group;
    int n_part, n_rows, row_pitch;   // rows per KV head: row = node*group + jj
    // chunk scores from per-tile logit sums (tile_sums == nullptr: none): extra workgroups of the same launch
    const float *tile_sums;   // [n_kv_heads][tile_sums_stride]
    float *scores;            // [n_kv_heads][n_chunks]
    int64_t tile_sums_stride, n_tokens, n_chunks;
    int chunk_size;           // multiple of 32
    float scale;
};
hipError_t launch_combine(const CombineParams &p, hipStream_t stream);

// ---- importance scores and top-k (scores_kernel.hip, topk_kernel.hip) -----------------------
struct ScoresParams {
    const uint16_t *q;        // bf16 [n_q_heads][128]
    const uint16_t *k;
    float *scores;            // [n_kv_heads][n_chunks]
    int64_t stride_head, stride_token;
    int64_t n_tokens;
    int64_t n_chunks;
    int n_q_heads, n_kv_heads, group;
    int chunk_size;
    float scale;
};
hipError_t launch_scores(const ScoresParams &p, hipStream_t stream);

struct TopkParams {
    const float *scores;      // [n_kv_heads][n_chunks]
    int32_t *idx_out;         // [n_kv_heads][n_sink + k]
    int n_kv_heads, n_chunks, n_sink, k;
};
hipError_t launch_topk(const TopkParams &p, hipStream_t stream);

// ---- cache maintenance (cache_kernels.hip) ------------------------------------------------------
struct AppendParams {
    uint16_t *k, *v;          // cache buffers (written)
    const uint16_t *k_tree, *v_tree;   // bf16 [n_tree][n_kv_heads][128]
    int64_t stride_head, stride_token;
    int64_t n_tokens;         // tokens cached before the append
    int n_kv_heads, n_accepted;
    int32_t accepted[kMaxTree];
};
hipError_t launch_append(const AppendParams &p, hipStream_t stream);
hipError_t launch_admit(int32_t *chunk_idx, int n_kv_heads, int n_sel, int n_sink, int base_chunk, int first_new_chunk, int n_new,
                        hipStream_t stream);

struct GatherParams {
    const uint16_t *k, *v;
    const int32_t *chunk_idx; // [n_kv_heads][n_sel]
    uint16_t *k_out, *v_out;  // [n_kv_heads][n_sel * chunk_size][128]
    int64_t stride_head, stride_token;
    int64_t n_tokens;
    int n_kv_heads, n_sel, chunk_size;
};
hipError_t launch_gather(const GatherParams &p, hipStream_t stream);

struct KsumParams {
    const uint16_t *k;
    float *ksum;              // element (h, c, x) at h*ksum_stride_head + c*128 + x
    int64_t stride_head, stride_token, ksum_stride_head;
    int64_t n_tokens, chunk_begin, chunk_end;
    int n_kv_heads, chunk_size;
};
hipError_t launch_ksum(const KsumParams &p, hipStream_t stream);

struct SumScoresParams {
    const float *ksum;
    const uint16_t *q;        // bf16 [n_q_heads][128]
    float *scores;            // [n_kv_heads][n_chunks]
    int64_t ksum_stride_head, n_tokens, n_chunks;
    int n_kv_heads, group, chunk_size;
    float scale;
};
hipError_t launch_sum_scores(const SumScoresParams &p, hipStream_t stream);

// ---- penalized probabilities and pool sampling (sampling_kernels.hip) -----------------------------
struct PenaltyParams {
    const float *logits;      // fp32 [n_rows][vocab]
    float *probs;             // fp32 [n_rows][vocab]
    const int32_t *window;    // device int32 [n_window]: ids of the tokens in the penalty window
    float *stats;             // [n_rows][n_slices][2]: per-slice max (exp2 domain) and sum of exponentials
    int64_t vocab;
    int n_rows, n_slices, n_window;
    float k_plain, k_window;  // log2(e) / t  and  log2(e) / (t * theta)
};
int sampling_slices(int64_t vocab);
hipError_t launch_penalized_probs(const PenaltyParams &p, hipStream_t stream);

enum { kSampleFull = 0, kSampleMinP = 1, kSampleTopP = 2, kSampleEta = 3 };
struct SampleParams {
    const float *probs;       // fp32 [n_rows][vocab]
    const float *u;           // fp32 [n_rows], uniform in [0, 1)
    int32_t *tokens;          // [n_rows]
    float *pool_threshold;    // [n_rows] or nullptr
    float *pool_mass;         // [n_rows] or nullptr
    int64_t vocab;
    int n_rows, method;
    float param, param2;
};
hipError_t launch_sample(const SampleParams &p, hipStream_t stream);

// ---- streaming-read probe (stream_read_kernel.hip) ----------------------------------------------
hipError_t launch_stream_read(const void *src, int64_t n_vec, uint32_t *sink, hipStream_t stream);

}  // namespace ts
