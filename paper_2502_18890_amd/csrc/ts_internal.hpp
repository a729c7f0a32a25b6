// Host <-> kernel parameter blocks and launcher declarations (internal to the library).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ts {

// ---- tree verification (verify_kernel.hip) -------------------------------------------------
struct VerifyParams {
    const uint16_t *q;        // bf16 [n_tree][n_q_heads][128]
    const uint16_t *k;        // cache keys
    const uint16_t *v;        // cache values
    const uint16_t *k_tree;   // bf16 [n_tree][n_kv_heads][128]
    const uint16_t *v_tree;
    float *ws_o;              // [n_kv_heads][n_split+1][n_rows_pad][128]
    float *ws_ml;             // [n_kv_heads][n_split+1][n_rows_pad][2]  (max in exp2 domain, sum)
    int64_t stride_head, stride_token;
    int64_t n_tokens;
    int64_t split_len;        // cached tokens per split, multiple of 32
    int n_split;              // number of cache splits (0 if the cache is empty); index n_split = tree
    int n_q_heads, n_kv_heads, group, n_tree;
    int n_rows;               // group * n_tree
    int n_rows_pad;           // row pitch of the workspace
    float scale_log2;         // scale * log2(e)
    uint64_t anc[64];         // anc[i] bit u set iff tree node u is i or an ancestor of i
};
int verify_rows_capacity(int n_rows);   // 0 if too many rows
hipError_t launch_verify(const VerifyParams &p, hipStream_t stream);        // K/V staged through registers
hipError_t launch_verify_dma(const VerifyParams &p, hipStream_t stream, int variant);   // K/V loaded straight into LDS

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
    int segs_per_chunk;       // chunk_size / 16: a 16-lane row handles one 16-token segment
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

}  // namespace ts
