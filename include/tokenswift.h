/*
 * tokenswift.h -- C ABI of the MI355X (gfx950) decode-attention hot path of TokenSwift
 * (arXiv 2502.18890): importance scoring and top-k selection for the dynamic partial KV
 * cache, attention over that partial cache, and tree-masked verification attention over
 * the full cache.
 *
 * General conventions
 *   - Every pointer is a DEVICE pointer unless its comment says HOST.  The caller owns all
 *     buffers, including the workspace; the library never allocates or frees device memory and
 *     keeps no state between calls other than the overrides of ts_tune_set and, per device, its
 *     number of compute units (read once).
 *   - bf16 arrays are passed as `const void*` (2-byte elements, IEEE bfloat16 bit patterns).
 *     Outputs are fp32.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work: outputs are valid once the stream has reached the call.  No call
 *     synchronises.
 *   - Every function returns a ts_status.  Arguments are validated on the host before
 *     anything is launched; on any error nothing has been enqueued.  Device-resident index
 *     arrays (chunk_idx) are NOT validated: chunk ids outside [0, n_chunks) are a caller
 *     error with undefined results.
 *   - head_dim is 128.  Rows of K and V (one token of one head) must be 16-byte aligned and
 *     contiguous in the head dimension; heads and tokens are addressed through element
 *     strides, so head-major [H_kv][N][128] and token-major [N][H_kv][128] caches both work.
 *   - One call handles one layer, batch 1.
 */
#ifndef TOKENSWIFT_H
#define TOKENSWIFT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    TS_OK = 0,
    TS_ERR_NULL = -1,        /* a required pointer is NULL */
    TS_ERR_SHAPE = -2,       /* sizes are inconsistent or out of range (N < 1, empty selection, ...) */
    TS_ERR_UNSUPPORTED = -3, /* valid in principle, outside what the kernels cover (head_dim != 128, ...) */
    TS_ERR_TREE = -4,        /* parent[] is not a forest in topological order */
    TS_ERR_WORKSPACE = -5,   /* workspace missing or smaller than ts_workspace_bytes() */
    TS_ERR_HIP = -6,         /* a HIP runtime call or kernel launch failed */
    TS_ERR_ALIGN = -7        /* a pointer or stride breaks the 16-byte row alignment */
} ts_status;

/* Limits of the kernels. */
#define TS_HEAD_DIM 128
#define TS_MAX_TREE 128       /* tree nodes per call (one 128-bit ancestor mask per node) */
#define TS_MAX_GROUP 8        /* query heads per KV head */
#define TS_MAX_CHUNKS (1 << 20)  /* chunks per KV head that ts_topk_chunks can rank; also the longest chunk list (n_sel) */
#define TS_MAX_TOPK 8192      /* chunks per KV head that ts_topk_chunks can select (k) */
#define TS_MAX_STRIDE_TOKEN (1 << 24) /* largest stride_token, in elements (32 MiB between token rows) */
#define TS_STATIC_SCRATCH_BYTES (4 << 20) /* fixed scratch of ts_partial_kv_attn_static, per GPU */

/* One layer's KV cache, as the paper's C_full (Alg. 1): n_tokens cached (key, value) pairs
 * for each of n_kv_heads heads.  Element (h, t, x) of K lives at
 * ((const bf16*)k)[h*stride_head + t*stride_token + x]; V uses the same strides. */
typedef struct {
    const void *k;          /* bf16 */
    const void *v;          /* bf16; may be NULL for ts_chunk_scores */
    int64_t n_tokens;       /* N >= 1 (ts_tree_verify_attn also accepts 0: tree tokens only) */
    int32_t n_kv_heads;
    int32_t head_dim;       /* must be TS_HEAD_DIM */
    int64_t stride_head;    /* elements; multiple of 8 */
    int64_t stride_token;   /* elements; multiple of 8, >= head_dim, <= TS_MAX_STRIDE_TOKEN */
} ts_kv_view;

enum { TS_OP_PARTIAL_ATTN = 1, TS_OP_TREE_VERIFY = 2, TS_OP_TREE_VERIFY_SCORED = 3 };

/*
 * All calls enqueue kernels on the caller's stream and return; none allocates, synchronises or
 * copies, so a sequence of them can be captured in a HIP graph.  The first call of some shapes sets
 * a kernel attribute (dynamic LDS above 64 KiB): run each shape once before capturing it.
 */

/* Text for a ts_status (static storage, never NULL). */
const char *ts_strerror(int status);

/* ABI version: major*10000 + minor*100 + patch. */
int ts_version(void);

/*
 * Bytes of device workspace that the split-K attention calls need for the given shape
 * (0 on invalid arguments).  op is TS_OP_PARTIAL_ATTN (n_sel, chunk_size used; n_tree ignored)
 * or TS_OP_TREE_VERIFY / TS_OP_TREE_VERIFY_SCORED (n_tree used; n_sel, chunk_size ignored).  The workspace holds the
 * per-split softmax partials (running max, sum of exponentials, unnormalised output) that a
 * second kernel merges (for TS_OP_TREE_VERIFY_SCORED also one logit sum per KV head and 32-key tile
 * of the cache); its contents are scratch and need no initialisation.
 */
size_t ts_workspace_bytes(int op, int n_q_heads, int n_kv_heads, int64_t n_tokens, int n_tree,
                          int n_sel, int chunk_size);

/*
 * Importance scores of the cached keys (Sec. 3.3, "Importance Score of KV pairs", Eq. 2),
 * averaged per chunk of `chunk_size` consecutive tokens:
 *
 *   scores[h][c] = scale * mean_{t in chunk c} sum_{j = h*g}^{(h+1)*g - 1} q[j] . K[h][t]
 *
 * with g = n_q_heads / kv->n_kv_heads (the GQA form of Eq. 2: the g query heads of a group
 * are summed against the one shared key; g = 1 is plain Q K^T).  A short last chunk averages
 * over its valid tokens.  chunk_size = 1 gives the per-token score of the paper.
 *   q       bf16 [n_q_heads][128]: the query token that ranks the cache
 *   scores  fp32 [n_kv_heads][ceil(N / chunk_size)]
 * chunk_size: 1..1024.  Errors: NULL pointers, n_q_heads not a multiple of n_kv_heads,
 * g > TS_MAX_GROUP, head_dim != 128, N < 1.
 */
int ts_chunk_scores(const ts_kv_view *kv, const void *q, int n_q_heads, int chunk_size,
                    float scale, float *scores, void *stream);

/*
 * Chunk selection for the partial cache C_p = {C_full[0:|S|], Top-K_{|B|-|S|}(C_full)}
 * (Alg. 1, prefill of C_p and "Dynamic KV Cache Update"; Sec. 3.3, "Dynamic KV Cache Updates"):
 * per KV head, idx_out = [0, .., n_sink_chunks-1] followed by the k highest-scoring chunks
 * among n_sink_chunks .. n_chunks-1, in order of decreasing score.  Equal scores rank by
 * lower chunk index (-0 equals +0); NaN scores rank below every number, by index.
 *   scores   fp32 [n_kv_heads][n_chunks]
 *   idx_out  int32 [n_kv_heads][n_sink_chunks + k]
 * Errors: n_chunks < 1 or > TS_MAX_CHUNKS, k > TS_MAX_TOPK, n_sink_chunks < 0, k < 0,
 * n_sink_chunks + k > n_chunks, n_sink_chunks + k == 0.
 */
int ts_topk_chunks(const float *scores, int n_kv_heads, int n_chunks, int n_sink_chunks, int k,
                   int32_t *idx_out, void *stream);

/*
 * Attention of the drafting forward pass over the partial cache (Alg. 1, "Multi-token
 * Parallel Generation"): one query token per head, softmax(scale * q K_sel^T) V_sel over
 * exactly the tokens of the listed chunks (chunk c = tokens [c*chunk_size,
 * min(N, (c+1)*chunk_size))).  The chunks are read in place through the index list; nothing
 * is copied.  A chunk listed twice counts twice.
 *   q          bf16 [n_q_heads][128]
 *   chunk_idx  int32 [n_kv_heads][n_sel]   (device; as written by ts_topk_chunks)
 *   out        fp32 [n_q_heads][128]
 *   lse        fp32 [n_q_heads], natural-log sum of exponentials of the scaled logits; nullable
 *   workspace  >= ts_workspace_bytes(TS_OP_PARTIAL_ATTN, ...) bytes, 256-byte aligned
 * chunk_size: multiple of 16, 16..1024.  scale must be positive and below 2e38, so that scale * log2(e)
 * is finite (TS_ERR_UNSUPPORTED otherwise).  Errors as above plus n_sel < 1 (TS_ERR_SHAPE) and
 * n_sel > TS_MAX_CHUNKS (TS_ERR_UNSUPPORTED).
 */
int ts_partial_kv_attn(const ts_kv_view *kv, const void *q, int n_q_heads,
                       const int32_t *chunk_idx, int n_sel, int chunk_size, float scale,
                       float *out, float *lse, void *workspace, size_t workspace_bytes,
                       void *stream);

/*
 * ts_partial_kv_attn for callers that cannot provide (or allocate) a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical results; the split partials go to a fixed array of TS_STATIC_SCRATCH_BYTES bytes that
 * lives in the library's device image (each GPU the library runs on holds it until the process ends).
 * The call allocates and frees nothing.  Its first call on a device looks up that device's address
 * of the array (once; do this outside a graph capture).
 *   - Shapes whose partials exceed the array return TS_ERR_WORKSPACE and enqueue nothing:
 *     ts_workspace_bytes(TS_OP_PARTIAL_ATTN, ...) <= TS_STATIC_SCRATCH_BYTES must hold (the five workloads of
 *     the benchmark need 0.02 to 1.4 MB).
 *   - Every call on a GPU shares that GPU's array: calls that may overlap on one GPU (different
 *     streams, or threads) race on it.  Calls on one stream are ordered and safe.  Nothing in the array
 *     has to start at zero; it keeps the last call's partials.
 * Errors otherwise as for ts_partial_kv_attn; TS_ERR_UNSUPPORTED for a device index >= 64.
 */
int ts_partial_kv_attn_static(const ts_kv_view *kv, const void *q, int n_q_heads,
                              const int32_t *chunk_idx, int n_sel, int chunk_size, float scale,
                              float *out, float *lse, void *stream);

/*
 * Verification attention of the draft-token tree over the full cache (Alg. 1, "Parallel
 * Verification"; App. E): row (node i, query head j) attends to every cached token of KV
 * head j/g and to tree node u iff u == i or u is an ancestor of i.
 *   q_tree          bf16 [n_tree][n_q_heads][128]
 *   k_tree, v_tree  bf16 [n_tree][n_kv_heads][128]  (keys/values of the tree tokens; the cache
 *                   holds accepted tokens only)
 *   parent          HOST int32 [n_tree]: parent[i] == -1 (root) or 0 <= parent[i] < i;
 *                   several roots are allowed.  Read during the call, not retained.
 *   out             fp32 [n_tree][n_q_heads][128]
 *   lse             fp32 [n_tree][n_q_heads]; nullable
 *   workspace       >= ts_workspace_bytes(TS_OP_TREE_VERIFY, ...) bytes, 256-byte aligned
 * n_tree: 1..TS_MAX_TREE.  kv->n_tokens may be 0 (then kv->k, kv->v may be NULL) and must be below 2^31.  scale must be
 * positive and below 2e38 (TS_ERR_UNSUPPORTED otherwise).
 * Errors: TS_ERR_TREE for a malformed parent array; the others as above.
 */
int ts_tree_verify_attn(const ts_kv_view *kv, const void *q_tree, int n_q_heads,
                        const void *k_tree, const void *v_tree, const int32_t *parent,
                        int n_tree, float scale, float *out, float *lse, void *workspace,
                        size_t workspace_bytes, void *stream);

/*
 * The same verification pass, which also leaves chunk importance scores of the cache (Eq. 2) for the
 * query of tree node 0:
 *   scores[h][c] = scale * mean over the tokens t of chunk c of sum_{j in group h} q_tree[0][j] . K[h][t],
 * i.e. what ts_chunk_scores returns for q = q_tree[0], at no extra pass over the keys: the rows of node 0
 * hold these products anyway.  Sec. 3.3 says that the scores are recomputed from query-key products; it
 * does not say of which forward pass or of which query.  Taking the verification pass and the query of
 * tree node 0 (the token the iteration starts from) is this library's reading; a caller that ranks the
 * cache with another query uses ts_chunk_scores or ts_chunk_scores_from_sums.
 *   scores      fp32 [n_kv_heads][ceil(N / chunk_size)]  (written; valid when the stream reaches the call)
 *   chunk_size  multiple of 32, 32..1024 (TS_ERR_UNSUPPORTED otherwise)
 *   workspace   >= ts_workspace_bytes(TS_OP_TREE_VERIFY_SCORED, ...) bytes, 256-byte aligned
 * kv->n_tokens must be >= 1 (TS_ERR_SHAPE).  Everything else as for ts_tree_verify_attn; out and lse are
 * the same as that call's.
 */
int ts_tree_verify_attn_scored(const ts_kv_view *kv, const void *q_tree, int n_q_heads,
                               const void *k_tree, const void *v_tree, const int32_t *parent,
                               int n_tree, float scale, int chunk_size, float *scores, float *out,
                               float *lse, void *workspace, size_t workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * Cache maintenance around the attention calls (Alg. 1: the update of C_full and the eviction
 * inside C_p at the end of each iteration, the "Dynamic KV Cache Update" step; Sec. 3.3
 * "Dynamic KV Cache Updates").
 * ------------------------------------------------------------------------------------- */

/*
 * Appends the accepted draft tokens to the full cache (Alg. 1, last step of the loop: "update
 * C_full"): for i < n_accepted, row kv->n_tokens + i of every KV head becomes the key/value
 * of tree node accepted[i].
 *   kv        the cache BEFORE the append (n_tokens = N); its k and v buffers are written and
 *             must have room for N + n_accepted tokens per head (capacity is the caller's)
 *   k_tree, v_tree  bf16 [n_tree][n_kv_heads][128]
 *   accepted  HOST pointer, int32 [n_accepted], each in [0, n_tree): the accepted path
 * n_tree, n_accepted: 1..TS_MAX_TREE.  kv->n_tokens may be 0.  The caller then uses N + n_accepted.
 * Errors: TS_ERR_TREE for an index outside [0, n_tree); the others as above.
 */
int ts_append_accepted(const ts_kv_view *kv, const void *k_tree, const void *v_tree, int n_tree,
                       const int32_t *accepted, int n_accepted, void *stream);

/*
 * When the partial cache must be rebuilt (Alg. 1, the condition guarding the "Dynamic KV Cache
 * Update" step: more than |B| - |S| tokens were added since the last rebuild at size e; Sec. 3.3:
 * new tokens replace the least important entries of C_p from position |B|-1 towards |S|, and
 * once they would pass |S| the importance scores are recomputed).  All sizes in tokens.
 * Returns 1 if a rebuild is due, 0 if not, TS_ERR_SHAPE for negative or inconsistent sizes.
 * Pure host arithmetic.
 */
int ts_refresh_due(int64_t n_tokens, int64_t n_tokens_at_refresh, int64_t budget_tokens, int64_t sink_tokens);

/*
 * Between rebuilds, newly generated tokens take the place of the least important entries of
 * C_p, from its last position towards the sink (Sec. 3.3).  At chunk granularity: base_chunk is the
 * chunk that receives the first token generated after the last rebuild (tokens at the rebuild /
 * chunk_size); chunk c >= base_chunk owns entry n_sel - 1 - (c - base_chunk) of every KV head's list
 * from the moment its first token exists (the list is ordered by decreasing importance, so its tail
 * holds the least important chunks).  The call admits chunks first_new_chunk .. first_new_chunk +
 * n_new_chunks - 1, in that order, per KV head:
 *   - c is not listed: it replaces the entry at its position (that chunk is evicted);
 *   - c is already listed among the non-sink entries (the partly filled last chunk, if the rebuild
 *     selected it; or c was admitted before): it trades places with the entry at its position and
 *     nothing is evicted; admitting a chunk again is therefore harmless;
 *   - c is one of the sink entries: nothing changes.
 * A list must never hold a chunk twice (ts_partial_kv_attn would count its keys twice in the
 * softmax); ts_topk_chunks writes duplicate-free lists and this call keeps them so.  Call it for the
 * chunks that received tokens, before the next drafting pass, so that every generated token is
 * visible to it; ts_partial_kv_attn clips a partly filled chunk to the cache's n_tokens.
 *   chunk_idx  device int32 [n_kv_heads][n_sel], as written by ts_topk_chunks (updated in place)
 * Errors (TS_ERR_SHAPE): first_new_chunk < base_chunk, n_new_chunks < 0, or first_new_chunk +
 * n_new_chunks - base_chunk > n_sel - n_sink_chunks (the new chunks would reach the sink: a rebuild
 * is due instead, which ts_refresh_due reports when it is given the rebuild size rounded down to a
 * chunk boundary, base_chunk * chunk_size).
 */
int ts_chunk_list_admit(int32_t *chunk_idx, int n_kv_heads, int n_sel, int n_sink_chunks, int base_chunk,
                        int first_new_chunk, int n_new_chunks, void *stream);

/*
 * Physical partial cache: copies the listed chunks into contiguous buffers, chunk j of head h
 * to rows j*chunk_size .. of k_out[h], v_out[h] (the paper rebuilds C_p as a buffer of its own;
 * ts_partial_kv_attn does not need this copy, it reads the chunks in place).
 *   k_out, v_out  bf16 [n_kv_heads][n_sel * chunk_size][128]; rows of a chunk past the end of
 *                 the cache are zero-filled
 * chunk_size: multiple of 16, 16..1024; 1 <= n_sel <= TS_MAX_CHUNKS.
 */
int ts_gather_chunks(const ts_kv_view *kv, const int32_t *chunk_idx, int n_sel, int chunk_size,
                     void *k_out, void *v_out, void *stream);

/*
 * Per-chunk key sums: ksum[h][c][x] = sum_{t in chunk c} K[h][t][x] (fp32), for chunks
 * chunk_begin <= c < chunk_end.  Eq. 2 is linear in the key, so the chunk score is a dot product
 * of the summed group query with this sum; a caller that refreshes the sums of the chunks it
 * appended to (only the last ones change) can rank the whole cache without re-reading it.
 *   ksum  fp32, element (h, c, x) at ksum[h*ksum_stride_head + c*128 + x]
 * Errors: chunk range outside [0, ceil(N / chunk_size)], chunk_size outside 1..1024.
 */
int ts_chunk_key_sums(const ts_kv_view *kv, int chunk_size, int64_t chunk_begin, int64_t chunk_end,
                      float *ksum, int64_t ksum_stride_head, void *stream);

/*
 * The scores of ts_chunk_scores, computed from the key sums instead of the keys:
 *   scores[h][c] = scale / |chunk c| * (sum_{j in group h} q[j]) . ksum[h][c]
 * (same value up to fp32 rounding order).  n_tokens is needed for the size of the last chunk.
 *   scores  fp32 [n_kv_heads][ceil(n_tokens / chunk_size)]
 */
int ts_chunk_scores_from_sums(const float *ksum, int64_t ksum_stride_head, int n_kv_heads,
                              int64_t n_tokens, const void *q, int n_q_heads, int chunk_size,
                              float scale, float *scores, void *stream);

/* ---------------------------------------------------------------------------------------
 * Penalized probabilities and sampling pools (Sec. 3.4 "Contextual Penalty", Eq. 3; App. D).
 * ------------------------------------------------------------------------------------- */

enum { TS_SAMPLE_FULL = 0, TS_SAMPLE_MIN_P = 1, TS_SAMPLE_TOP_P = 2, TS_SAMPLE_ETA = 3 };

/* Bytes of device workspace ts_penalized_probs needs (0 on invalid arguments). */
size_t ts_sampling_workspace_bytes(int n_rows, int64_t vocab);

/*
 * Eq. 3: probs[r][i] = softmax_i( logits[r][i] / (temperature * I_i) ), I_i = theta if token i occurs
 * in `window` (the ids of the most recent W generated tokens; repeats allowed, ids outside
 * [0, vocab) ignored), else 1.  As printed in the paper, the logit is divided whatever its sign.
 *   logits, probs  fp32 [n_rows][vocab], 16-byte aligned (may not alias)
 *   window         device int32 [n_window]; may be NULL when n_window == 0
 *   workspace      >= ts_sampling_workspace_bytes(n_rows, vocab) bytes, 256-byte aligned; scratch
 * temperature > 0, theta >= 1, both finite; 1 <= vocab <= 2^24; n_rows >= 1.
 */
int ts_penalized_probs(const float *logits, int n_rows, int64_t vocab, const int32_t *window,
                       int n_window, float temperature, float theta, float *probs, void *workspace,
                       size_t workspace_bytes, void *stream);

/*
 * Draws one token per row from a sampling pool of App. D with the renormalised probabilities.
 * The pool is {i : probs[r][i] >= tau_r}: TS_SAMPLE_FULL: every token; TS_SAMPLE_MIN_P: tau = param *
 * max_i probs[r][i] (param = p_base in (0, 1]); TS_SAMPLE_TOP_P: the largest tau whose pool still holds
 * mass >= param (param = p in (0, 1]): the most probable tokens whose mass reaches p, tokens tied
 * with the last one all kept; TS_SAMPLE_ETA: tau = min(param, param2 * exp(-h_r)) with h_r the entropy
 * (natural log) of row r (param = epsilon in (0, 1], param2 = alpha > 0).  param2 is ignored by the
 * other methods.  The draw inverts the pool's cumulative distribution, taken in order
 * of token id, at u[r]: the first pool token whose cumulative pool mass exceeds u[r] * pool mass.
 *   probs  fp32 [n_rows][vocab]; u  device fp32 [n_rows] in [0, 1) (clamped); tokens  int32 [n_rows]
 *   pool_threshold, pool_mass  fp32 [n_rows], nullable: tau_r and the pool's mass
 */
int ts_sample_tokens(const float *probs, int n_rows, int64_t vocab, int method, float param,
                     float param2, const float *u, int32_t *tokens, float *pool_threshold,
                     float *pool_mass, void *stream);

/*
 * Tuning hook (not needed for correct results): overrides a launch-geometry choice until
 * reset with value 0.  Names: "verify_splits" (number of cache splits per KV head);
 * "verify_variant" (1..3: alternative kernel shapes of the verification pass); "verify_kernel" (k > 0: the
 * k-th instantiation of the verification kernels wherever it can cover the call's query rows per KV head, the
 * default shape elsewhere: lets tests and measurements reach every instantiation).  Every setting
 * produces the same results up to rounding order.  Returns TS_OK, or TS_ERR_UNSUPPORTED for an
 * unknown name or a value the kernels cannot run.  The same setting is seen by ts_workspace_bytes,
 * so size the workspace after setting it.  This is the only mutable state of the library (process-wide,
 * atomic words: a concurrent call sees the old or the new value).
 */
int ts_tune_set(const char *name, int value);

/*
 * Measurement utility (no passage of the paper): enqueues ONLY the first of the two kernels of
 * ts_tree_verify_attn -- the one that streams the cache and leaves per-split partial results in the
 * workspace -- so that it can be timed alone for the roofline figure.  No output is produced (there are no
 * out / lse arguments); the workspace contents afterwards are scratch.  with_tile_sums != 0 runs the
 * variant of ts_tree_verify_attn_scored (size the workspace for TS_OP_TREE_VERIFY_SCORED then), else
 * that of ts_tree_verify_attn.  Arguments and errors otherwise as for those calls.
 */
int ts_bench_verify_split_kernel(const ts_kv_view *kv, const void *q_tree, int n_q_heads,
                                 const void *k_tree, const void *v_tree, const int32_t *parent,
                                 int n_tree, float scale, int with_tile_sums, void *workspace,
                                 size_t workspace_bytes, void *stream);

/*
 * Measurement utility (no passage of the paper): enqueues a kernel that reads `bytes` bytes at
 * `src` (device, 16-byte aligned, bytes a multiple of 16) exactly once with 128-bit loads and
 * does nothing else.  Timed over the cache buffers, it gives the read rate the memory system
 * sustains, the practical ceiling for the bandwidth-bound passes.  `sink` (device, 4 bytes,
 * caller-owned) is written only if the buffer's words fold to one particular value; its content
 * carries no meaning.  Returns TS_ERR_NULL, TS_ERR_SHAPE (size or alignment), TS_ERR_UNSUPPORTED
 * (more than 2^42 bytes), TS_ERR_HIP, else TS_OK.  Asynchronous on `stream`.
 */
int ts_stream_read_probe(const void *src, size_t bytes, uint32_t *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* TOKENSWIFT_H */
