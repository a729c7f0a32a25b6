/*
 * ts_oracle.c -- fp64 CPU oracle for the decode-attention hot path of TokenSwift.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the HIP
 * kernels are checked against.  It shares no code, header, table or helper with the
 * GPU library, and nothing in the product path may call it.
 *
 * What it defines (paper passages it follows):
 *   oracle_chunk_scores   Sec. 3.3 "Importance Score of KV pairs" and Eq. 2: the score of a
 *                         cached key of KV head i is the sum, over the g query heads of
 *                         that head's group, of Q_j . K_i (the key is not replicated).
 *                         Here the per-token score is averaged over each chunk of
 *                         `chunk` consecutive tokens (a short last chunk averages over
 *                         its valid tokens only); chunk = 1 is the paper's per-token score.
 *   oracle_topk_chunks    Sec. 3.3 "Dynamic KV Cache Updates" and Alg. 1 (prefill of the
 *                         partial cache and "Dynamic KV Cache Update"): the partial cache
 *                         is the first |S| entries followed by the |B|-|S| most important
 *                         of the others, in order of decreasing importance.
 *   oracle_partial_attn   Alg. 1 "Multi-token Parallel Generation" (the forward pass with
 *                         partial cache C_p): ordinary softmax attention of one query
 *                         token per head over exactly the keys that the chunk list names.
 *   oracle_tree_verify    Alg. 1 "Parallel Verification" and App. E (tree-based attention):
 *                         every tree token attends to the whole full cache and to those
 *                         tree tokens that are its predecessors in the tree, itself included.
 *   oracle_combine        log-sum-exp merge of attention partials over disjoint key sets
 *                         (an identity of softmax; used only to test the split-K design).
 *
 * All arithmetic is double.  Inputs are bf16 bit patterns (uint16) widened exactly.
 * There is no blocking, no running max, no split: each softmax is computed by the
 * textbook three passes (max, sum of exponentials, weighted sum) over its whole key set.
 * Threads (OpenMP) only distribute independent output rows.
 *
 * Parity pins (tests/test_oracle_pins.py): every function here is pinned by closed forms,
 * special cases that reduce to library routines, invariants and brute force.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_OK 0
#define ORACLE_ERR_ARG -1

static double bf16_to_f64(uint16_t bits)
{
    uint32_t u = ((uint32_t)bits) << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* dot product of two bf16 rows of length d, in double */
static double dot_bf16(const uint16_t *a, const uint16_t *b, int d)
{
    double s = 0.0;
    for (int x = 0; x < d; ++x) s += bf16_to_f64(a[x]) * bf16_to_f64(b[x]);
    return s;
}

/*
 * Eq. 2, averaged per chunk.
 *   q      [n_q_heads][d]           bf16
 *   k      element (h, t, x) at k[h*stride_head + t*stride_token + x], bf16
 *   scores [n_kv_heads][n_chunks]   double, n_chunks = ceil(n_tokens / chunk)
 * scores[h][c] = scale * (1/|chunk c|) * sum_{t in chunk c} sum_{j in group h} q_j . k_{h,t}
 */
int oracle_chunk_scores(const uint16_t *q, const uint16_t *k, int n_q_heads, int n_kv_heads,
                        int64_t n_tokens, int d, int64_t stride_head, int64_t stride_token,
                        int chunk, double scale, double *scores)
{
    if (!q || !k || !scores || n_q_heads < 1 || n_kv_heads < 1 || n_tokens < 1 || d < 1 ||
        chunk < 1 || n_q_heads % n_kv_heads != 0)
        return ORACLE_ERR_ARG;
    const int g = n_q_heads / n_kv_heads;
    const int64_t n_chunks = (n_tokens + chunk - 1) / chunk;
#pragma omp parallel for collapse(2) schedule(static)
    for (int h = 0; h < n_kv_heads; ++h) {
        for (int64_t c = 0; c < n_chunks; ++c) {
            const int64_t lo = c * chunk;
            const int64_t hi = (lo + chunk < n_tokens) ? lo + chunk : n_tokens;
            double total = 0.0;
            for (int64_t t = lo; t < hi; ++t) {
                const uint16_t *krow = k + h * stride_head + t * stride_token;
                double token_score = 0.0; /* Eq. 2 for this cached key */
                for (int j = h * g; j < (h + 1) * g; ++j)
                    token_score += dot_bf16(q + (int64_t)j * d, krow, d);
                total += token_score;
            }
            scores[(int64_t)h * n_chunks + c] = scale * total / (double)(hi - lo);
        }
    }
    return ORACLE_OK;
}

/* "a ranks strictly before b": higher score first, equal scores -> lower index first,
 * NaN after every number, NaNs among themselves by index.  -0 == +0 as for doubles. */
static int ranks_before(double sa, int64_t ia, double sb, int64_t ib)
{
    const int na = isnan(sa), nb = isnan(sb);
    if (na || nb) {
        if (na && nb) return ia < ib;
        return nb; /* the number ranks before the NaN */
    }
    if (sa > sb) return 1;
    if (sa < sb) return 0;
    return ia < ib;
}

/*
 * Alg. 1, construction of C_p = {C_full[0:|S|], Top-K_{|B|-|S|}(C_full)}, at chunk granularity.
 *   scores [n_kv_heads][n_chunks] double
 *   idx    [n_kv_heads][n_sink + k] int32:  0..n_sink-1, then the k best of the chunks
 *          n_sink..n_chunks-1 in order of decreasing score (ties -> lower index).
 * Selection by k rounds of "take the best not yet taken".
 */
int oracle_topk_chunks(const double *scores, int n_kv_heads, int64_t n_chunks, int n_sink, int k,
                       int32_t *idx)
{
    if (!scores || !idx || n_kv_heads < 1 || n_chunks < 1 || n_sink < 0 || k < 0 ||
        (int64_t)n_sink + k > n_chunks || n_sink + k < 1)
        return ORACLE_ERR_ARG;
    for (int h = 0; h < n_kv_heads; ++h) {
        const double *s = scores + (int64_t)h * n_chunks;
        int32_t *out = idx + (int64_t)h * (n_sink + k);
        unsigned char *taken = (unsigned char *)calloc((size_t)n_chunks, 1);
        if (!taken) return ORACLE_ERR_ARG;
        for (int i = 0; i < n_sink; ++i) out[i] = i;
        for (int r = 0; r < k; ++r) {
            int64_t best = -1;
            for (int64_t c = n_sink; c < n_chunks; ++c) {
                if (taken[c]) continue;
                if (best < 0 || ranks_before(s[c], c, s[best], best)) best = c;
            }
            taken[best] = 1;
            out[n_sink + r] = (int32_t)best;
        }
        free(taken);
    }
    return ORACLE_OK;
}

/* Softmax attention of one query row over an explicit list of key/value rows.
 * keys[i], vals[i] point at bf16 rows of length d.  Three plain passes. */
static void attend_rows(const uint16_t *qrow, const uint16_t *const *keys,
                        const uint16_t *const *vals, int64_t n_keys, int d, double scale,
                        double *logits /* scratch [n_keys] */, double *out /* [d] */, double *lse)
{
    double m = -INFINITY;
    for (int64_t i = 0; i < n_keys; ++i) {
        logits[i] = scale * dot_bf16(qrow, keys[i], d);
        if (logits[i] > m) m = logits[i];
    }
    double denom = 0.0;
    for (int64_t i = 0; i < n_keys; ++i) denom += exp(logits[i] - m);
    for (int x = 0; x < d; ++x) out[x] = 0.0;
    for (int64_t i = 0; i < n_keys; ++i) {
        const double p = exp(logits[i] - m) / denom;
        for (int x = 0; x < d; ++x) out[x] += p * bf16_to_f64(vals[i][x]);
    }
    if (lse) *lse = m + log(denom);
}

/*
 * Alg. 1 "Multi-token Parallel Generation": attention of one query token per head over the
 * partial cache.
 *   chunk_idx [n_kv_heads][n_sel] int32: chunk c names tokens [c*chunk, min(N,(c+1)*chunk)).
 *   out [n_q_heads][d] double, lse [n_q_heads] double (nullable).
 * A chunk listed twice contributes its keys twice.
 */
int oracle_partial_attn(const uint16_t *q, const uint16_t *k, const uint16_t *v, int n_q_heads,
                        int n_kv_heads, int64_t n_tokens, int d, int64_t stride_head,
                        int64_t stride_token, const int32_t *chunk_idx, int n_sel, int chunk,
                        double scale, double *out, double *lse)
{
    if (!q || !k || !v || !chunk_idx || !out || n_q_heads < 1 || n_kv_heads < 1 ||
        n_tokens < 1 || d < 1 || n_sel < 1 || chunk < 1 || n_q_heads % n_kv_heads != 0)
        return ORACLE_ERR_ARG;
    const int g = n_q_heads / n_kv_heads;
    const int64_t n_chunks = (n_tokens + chunk - 1) / chunk;
    for (int h = 0; h < n_kv_heads; ++h)
        for (int i = 0; i < n_sel; ++i) {
            const int32_t c = chunk_idx[(int64_t)h * n_sel + i];
            if (c < 0 || c >= n_chunks) return ORACLE_ERR_ARG;
        }
    int rc = ORACLE_OK;
#pragma omp parallel for schedule(static)
    for (int j = 0; j < n_q_heads; ++j) {
        const int h = j / g;
        const int64_t cap = (int64_t)n_sel * chunk;
        const uint16_t **keys = (const uint16_t **)malloc(sizeof(*keys) * (size_t)cap);
        const uint16_t **vals = (const uint16_t **)malloc(sizeof(*vals) * (size_t)cap);
        double *logits = (double *)malloc(sizeof(double) * (size_t)cap);
        if (!keys || !vals || !logits) {
            rc = ORACLE_ERR_ARG;
        } else {
            int64_t n_keys = 0;
            for (int i = 0; i < n_sel; ++i) {
                const int64_t c = chunk_idx[(int64_t)h * n_sel + i];
                const int64_t lo = c * chunk;
                const int64_t hi = (lo + chunk < n_tokens) ? lo + chunk : n_tokens;
                for (int64_t t = lo; t < hi; ++t) {
                    keys[n_keys] = k + h * stride_head + t * stride_token;
                    vals[n_keys] = v + h * stride_head + t * stride_token;
                    ++n_keys;
                }
            }
            attend_rows(q + (int64_t)j * d, keys, vals, n_keys, d, scale, logits,
                        out + (int64_t)j * d, lse ? lse + j : NULL);
        }
        free(keys);
        free(vals);
        free(logits);
    }
    return rc;
}

/* parent[] must be a forest in topological order: parent[i] == -1 or 0 <= parent[i] < i */
static int tree_ok(const int32_t *parent, int n_tree)
{
    for (int i = 0; i < n_tree; ++i)
        if (parent[i] < -1 || parent[i] >= i) return 0;
    return 1;
}

/*
 * Alg. 1 "Parallel Verification" with the mask of App. E: row (node i, query head j) attends to every cache
 * token of KV head j/g and to tree node u iff u == i or u is an ancestor of i.
 *   q_tree [n_tree][n_q_heads][d], k_tree/v_tree [n_tree][n_kv_heads][d], bf16
 *   parent [n_tree] int32
 *   Row selection: if n_rows >= 0, only rows (row_node[r], row_head[r]), r < n_rows, are
 *   computed and out is [n_rows][d]; if n_rows < 0, all rows, out is [n_tree][n_q_heads][d].
 *   lse laid out like out without the d axis (nullable).
 * n_tokens may be 0 (tree tokens only).
 */
int oracle_tree_verify(const uint16_t *q_tree, const uint16_t *k, const uint16_t *v,
                       const uint16_t *k_tree, const uint16_t *v_tree, const int32_t *parent,
                       int n_tree, int n_q_heads, int n_kv_heads, int64_t n_tokens, int d,
                       int64_t stride_head, int64_t stride_token, double scale,
                       const int32_t *row_node, const int32_t *row_head, int64_t n_rows,
                       double *out, double *lse)
{
    if (!q_tree || !k_tree || !v_tree || !parent || !out || n_tree < 1 || n_q_heads < 1 ||
        n_kv_heads < 1 || n_tokens < 0 || d < 1 || n_q_heads % n_kv_heads != 0)
        return ORACLE_ERR_ARG;
    if (n_tokens > 0 && (!k || !v)) return ORACLE_ERR_ARG;
    if (!tree_ok(parent, n_tree)) return ORACLE_ERR_ARG;
    if (n_rows >= 0 && (!row_node || !row_head)) return ORACLE_ERR_ARG;
    const int g = n_q_heads / n_kv_heads;
    const int64_t total = (n_rows >= 0) ? n_rows : (int64_t)n_tree * n_q_heads;
    for (int64_t r = 0; r < total && n_rows >= 0; ++r)
        if (row_node[r] < 0 || row_node[r] >= n_tree || row_head[r] < 0 ||
            row_head[r] >= n_q_heads)
            return ORACLE_ERR_ARG;
    int rc = ORACLE_OK;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t r = 0; r < total; ++r) {
        const int i = (n_rows >= 0) ? row_node[r] : (int)(r / n_q_heads);
        const int j = (n_rows >= 0) ? row_head[r] : (int)(r % n_q_heads);
        const int h = j / g;
        const int64_t cap = n_tokens + n_tree;
        const uint16_t **keys = (const uint16_t **)malloc(sizeof(*keys) * (size_t)cap);
        const uint16_t **vals = (const uint16_t **)malloc(sizeof(*vals) * (size_t)cap);
        double *logits = (double *)malloc(sizeof(double) * (size_t)cap);
        if (!keys || !vals || !logits) {
            rc = ORACLE_ERR_ARG;
        } else {
            int64_t n_keys = 0;
            for (int64_t t = 0; t < n_tokens; ++t) {
                keys[n_keys] = k + h * stride_head + t * stride_token;
                vals[n_keys] = v + h * stride_head + t * stride_token;
                ++n_keys;
            }
            /* walk from node i to its root: i itself, its parent, its grandparent, ... */
            for (int u = i; u != -1; u = parent[u]) {
                keys[n_keys] = k_tree + ((int64_t)u * n_kv_heads + h) * d;
                vals[n_keys] = v_tree + ((int64_t)u * n_kv_heads + h) * d;
                ++n_keys;
            }
            attend_rows(q_tree + ((int64_t)i * n_q_heads + j) * d, keys, vals, n_keys, d, scale,
                        logits, out + r * d, lse ? lse + r : NULL);
        }
        free(keys);
        free(vals);
        free(logits);
    }
    return rc;
}

/*
 * Merge of n_parts attention partials over disjoint key sets.  Partial p carries
 *   m[p]  = max logit of its keys, l[p] = sum exp(logit - m[p]), o[p][d] = sum exp(logit - m[p]) * v.
 * A partial with no keys is given as m = -inf, l = 0 and is ignored.
 * out[d] = attention over the union; lse (nullable) = log-sum-exp over the union.
 */
int oracle_combine(const double *m, const double *l, const double *o, int n_parts, int d,
                   double *out, double *lse)
{
    if (!m || !l || !o || !out || n_parts < 1 || d < 1) return ORACLE_ERR_ARG;
    double mstar = -INFINITY;
    for (int p = 0; p < n_parts; ++p)
        if (l[p] > 0.0 && m[p] > mstar) mstar = m[p];
    if (mstar == -INFINITY) return ORACLE_ERR_ARG;
    double lstar = 0.0;
    for (int x = 0; x < d; ++x) out[x] = 0.0;
    for (int p = 0; p < n_parts; ++p) {
        if (!(l[p] > 0.0)) continue;
        const double w = exp(m[p] - mstar);
        lstar += l[p] * w;
        for (int x = 0; x < d; ++x) out[x] += o[(int64_t)p * d + x] * w;
    }
    for (int x = 0; x < d; ++x) out[x] /= lstar;
    if (lse) *lse = mstar + log(lstar);
    return ORACLE_OK;
}
