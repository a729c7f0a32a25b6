// C ABI of the library: argument validation, launch-geometry choice, workspace carve-up.
// All validation happens on the host before anything is enqueued.
#include <string.h>
#include <mutex>

#include "../../include/tokenswift.h"
#include "ts_internal.hpp"

namespace {

// The only state the library keeps: launch-geometry overrides (ts_tune_set) and, per device, the
// number of compute units, read once.  Both are plain atomics: a reader sees the old or the new value.
struct Tuning {
    std::atomic<int> verify_splits{0};     // 0 = heuristic
    std::atomic<int> verify_variant{0};    // 0 = default kernel shapes; 1..3 = alternatives (see verify_shape)
    std::atomic<int> verify_kernel{0};     // 0 = by shape; k > 0 = kernel id k-1 where it can cover the rows (else by shape)
} g_tune;

// Compute units of the current device (256 on a whole MI355X, fewer on a partitioned one): the split
// heuristic fills exactly one resident round of workgroups.  Falls back to 256 if the query fails.
int device_cus()
{
    constexpr int kMaxDev = 64;
    static std::atomic<int> cached[kMaxDev];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (dev >= 0 && dev < kMaxDev) {
        const int c = cached[dev].load(std::memory_order_relaxed);
        if (c > 0) return c;
    }
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1) cus = 256;
    if (dev >= 0 && dev < kMaxDev) cached[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

// ---- the allocation-free entry point's scratch ---------------------------------------------------
// A fixed device array stands in for the caller's workspace.  Its name is a host-side stand-in, not a
// device address: host code uses the per-device pointer that hipGetSymbolAddress returns (each GPU
// holds its own copy of the array at its own address), never the name.
constexpr size_t kScratchBytes = (size_t)TS_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxScratchDevices = 64;
std::mutex g_scratch_lock;
void *g_scratch_ptr[kMaxScratchDevices];   // device address of `scratch` on each device, looked up on first use

int scratch_of_current_device(void **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return TS_ERR_HIP;
    if (dev < 0 || dev >= kMaxScratchDevices) return TS_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> hold(g_scratch_lock);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return TS_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return TS_OK;
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_view(const ts_kv_view *kv, bool need_v, bool allow_empty)
{
    if (!kv) return TS_ERR_NULL;
    if (kv->head_dim != TS_HEAD_DIM) return TS_ERR_UNSUPPORTED;
    if (kv->n_kv_heads < 1) return TS_ERR_SHAPE;
    if (kv->n_kv_heads > 65535) return TS_ERR_UNSUPPORTED;   // heads are a grid dimension
    if (kv->n_tokens < 0 || (kv->n_tokens == 0 && !allow_empty)) return TS_ERR_SHAPE;
    if (kv->n_tokens == 0) return TS_OK;
    if (!kv->k || (need_v && !kv->v)) return TS_ERR_NULL;
    if (kv->stride_token < TS_HEAD_DIM || kv->stride_head < 0) return TS_ERR_SHAPE;
    // the attention kernels address the 32 rows of a tile with 32-bit byte offsets
    if (kv->stride_token > TS_MAX_STRIDE_TOKEN) return TS_ERR_UNSUPPORTED;
    if ((kv->stride_token % 8) != 0 || (kv->stride_head % 8) != 0) return TS_ERR_ALIGN;
    if (!aligned16(kv->k) || (need_v && !aligned16(kv->v))) return TS_ERR_ALIGN;
    return TS_OK;
}

int check_heads(int n_q_heads, int n_kv_heads, int *group)
{
    if (n_q_heads < 1 || n_kv_heads < 1 || n_q_heads % n_kv_heads != 0) return TS_ERR_SHAPE;
    *group = n_q_heads / n_kv_heads;
    if (*group > TS_MAX_GROUP) return TS_ERR_UNSUPPORTED;
    return TS_OK;
}

// ---- geometry of the verification pass ------------------------------------------------------
struct VerifyPlan {
    ts::VerifyShape shape;
    int n_rows, n_rows_pad, n_split;
    int64_t split_len;
    size_t ml_offset, tile_offset, bytes;   // tile_offset: per-tile logit sums of the scored variant (0 bytes otherwise)
    int64_t n_tiles;
};

// Splits of the cache: as many workgroups as the chip holds at once (so that the grid runs as
// one resident wave with every CU's latency-hiding slots full), but few enough that the fp32
// partials (520 B per row and split) stay a small fraction of the K/V bytes (512 B per token).
bool plan_verify(int n_q_heads, int n_kv_heads, int64_t n_tokens, int n_tree, bool scored, VerifyPlan *pl)
{
    const int group = n_q_heads / n_kv_heads;
    pl->n_rows = group * n_tree;
    pl->n_rows_pad = (pl->n_rows + 15) / 16 * 16;
    if (!ts::verify_shape(pl->n_rows, n_kv_heads, n_tokens, g_tune.verify_variant.load(std::memory_order_relaxed), &pl->shape)) return false;
    if (const int forced = g_tune.verify_kernel.load(std::memory_order_relaxed)) {
        const ts::VerifyKernelInfo info = ts::verify_kernel_info(forced - 1);
        if (info.max_rows >= pl->n_rows) pl->shape = ts::VerifyShape{forced - 1, (pl->n_rows + 31) / 32 * 32, info.wg_per_cu};
        if (info.max_rows >= pl->n_rows && forced - 1 <= ts::kNarrow_32) pl->shape.rows_per_wg = info.max_rows;
    }
    int n_split = 0;
    int64_t split_len = 32;
    if (n_tokens > 0) {
        const int row_tiles = (pl->n_rows + pl->shape.rows_per_wg - 1) / pl->shape.rows_per_wg;
        const int64_t per_split = (int64_t)n_kv_heads * row_tiles;          // workgroups per split index
        // - 1: the tree split.  Not for the two-wavefront 16x16x32 kernel: its tree workgroups are over in a
        // few microseconds, so letting them (and the cache workgroups that then start late) run in slots that
        // free up early costs less than leaving one slot in 32 idle for the whole pass (257 vs 260 us at 100K).
        int64_t want = (int64_t)device_cus() * pl->shape.wg_per_cu / per_split - (pl->shape.kernel_id == ts::kNarrow_32 ? 0 : 1);
        const int64_t cap_traffic = (n_tokens * 512 / 4) / ((int64_t)pl->n_rows_pad * 520) + 1;  // partials <= 1/4 of K/V
        if (want > cap_traffic) want = cap_traffic;
        const int forced = g_tune.verify_splits.load(std::memory_order_relaxed);
        if (forced > 0) want = forced;
        const int64_t max_split = (n_tokens + 31) / 32;
        if (want > max_split) want = max_split;
        if (want < 1) want = 1;
        split_len = ((n_tokens + want - 1) / want + 31) / 32 * 32;
        n_split = (int)((n_tokens + split_len - 1) / split_len);
    }
    pl->n_split = n_split;
    pl->split_len = split_len;
    const size_t rows_total = (size_t)n_kv_heads * (n_split + 1) * pl->n_rows_pad;
    pl->ml_offset = round_up(rows_total * TS_HEAD_DIM * sizeof(float), 256);
    pl->tile_offset = pl->ml_offset + round_up(rows_total * 2 * sizeof(float), 256);
    pl->n_tiles = (n_tokens + 31) / 32;
    pl->bytes = pl->tile_offset + (scored ? round_up((size_t)n_kv_heads * pl->n_tiles * sizeof(float), 256) : 0);
    return true;
}

struct PartialPlan {
    int segs_per_chunk, n_seg, n_part;
    size_t ml_offset, bytes;
};

void plan_partial(int n_q_heads, int n_kv_heads, int n_sel, int chunk_size, PartialPlan *pl)
{
    const int group = n_q_heads / n_kv_heads;
    pl->segs_per_chunk = chunk_size / 8;
    pl->n_seg = n_sel * pl->segs_per_chunk;
    pl->n_part = (pl->n_seg + 15) / 16;
    const size_t rows_total = (size_t)n_kv_heads * pl->n_part * group;
    pl->ml_offset = round_up(rows_total * TS_HEAD_DIM * sizeof(float), 256);
    pl->bytes = pl->ml_offset + round_up(rows_total * 2 * sizeof(float), 256);
}

// the attention kernels take row maxima before scaling the logits, and work with scale * log2(e), which
// must stay finite
bool scale_ok(float scale) { return scale > 0.f && scale < 2.0e38f; }

bool partial_chunk_ok(int chunk_size) { return chunk_size >= 16 && chunk_size <= 1024 && chunk_size % 16 == 0; }

}  // namespace

// Kernel shape by number of query rows per KV head.  Up to 32 rows the pass is purely HBM-bound
// and the 16x16x32 kernel with its small workgroups (many of them per CU) is used; beyond that
// the 32x32x16 kernel, in row tiles of at most 384 rows.  Defaults are the fastest measured
// shapes; variant 1..3 select alternatives where there are any (all produce the same results):
// 1 swaps the precision of the second product (fp16 where the default is bf16 + residual and
// the other way round), 2 and 3 other workgroup shapes.
bool ts::verify_shape(int n_rows, int n_kv_heads, int64_t n_tokens, int variant, VerifyShape *out)
{
    if (n_rows < 1 || n_rows > TS_MAX_GROUP * TS_MAX_TREE) return false;
    if (variant == 0 && n_rows <= 16) {
        *out = VerifyShape{kNarrow_16, 16, 5};
        return true;
    }
    if (variant == 0 && n_rows <= 32) {
        *out = VerifyShape{kNarrow_32, 32, 4};
        return true;
    }
    const int tiles = (n_rows + 383) / 384;
    const int r = ((n_rows + tiles - 1) / tiles + 31) / 32 * 32;   // rows per tile, balanced
    if (r <= 32) *out = variant == 2 ? VerifyShape{kWide_1x1b, 32, 2} : VerifyShape{kWide_1x1, 32, 3};
    else if (r <= 64) {
        if (variant == 1) *out = VerifyShape{kWide_1x2h, 64, 2};
        else if (variant == 2) *out = VerifyShape{kWide_1x2, 64, 2};
        else *out = VerifyShape{kWide_1x2k4, 64, 1};
    }
    else if (r <= 128) {
        // With 8 or more KV heads the pass draws the chip's full power (1400 W at 1.7-1.9 GHz for 100 rows on 32 heads x
        // 100K tokens), and the fp16 second product's smaller matrix work, with the address arithmetic saved by
        // unrolling over the ring's stages, is the fastest: two workgroups of four wavefronts per CU where each
        // workgroup's range is long (100 rows on 32 heads x 100K: 308 us against 345 with bf16 weights + residuals,
        // 325 with one workgroup of eight), one workgroup of two key groups x four wavefronts, with half the partials to
        // write and merge, where it is short (128 rows on 8 heads x 65K: whole call 71 us against 74).  With few heads
        // one workgroup of three key groups with bf16 weights is faster (96 rows on 2 heads x 16K: 14.9 us against 17.2).
        const bool many_heads = n_kv_heads >= 8;
        const bool long_ranges = n_tokens * n_kv_heads / 512 >= 4096;   // tokens per workgroup at two workgroups per CU
        if (variant == 1) *out = many_heads ? VerifyShape{kWide_1x4, 128, 2} : VerifyShape{kWide_1x4h, 128, 2};
        else if (variant == 2) *out = many_heads ? VerifyShape{kWide_1x4k3, 128, 1} : VerifyShape{kWide_1x4, 128, 2};
        else if (variant == 3) *out = many_heads && !long_ranges ? VerifyShape{kWide_1x4h, 128, 2} : VerifyShape{kWide_1x4k2h, 128, 1};
        else if (many_heads) *out = long_ranges ? VerifyShape{kWide_1x4h, 128, 2} : VerifyShape{kWide_1x4k2h, 128, 1};
        else *out = VerifyShape{kWide_1x4k3, 128, 1};
    } else if (r <= 256) {
        if (variant == 1) *out = VerifyShape{kWide_1x8, 256, 1};
        else if (variant == 2) *out = VerifyShape{kWide_2x4, 256, 1};
        else if (variant == 3) *out = VerifyShape{kWide_1x8h, 256, 1};
        else *out = VerifyShape{kWide_1x8h4, 256, 1};   // four stages: their offsets ride in the instructions (3 % over six stages)
    } else {
        if (variant == 1) *out = r <= 320 ? VerifyShape{kWide_1x10, 320, 1} : VerifyShape{kWide_1x12, 384, 1};
        else *out = r <= 320 ? VerifyShape{kWide_1x10h, 320, 1} : VerifyShape{kWide_1x12h, 384, 1};
    }
    out->rows_per_wg = r;
    return true;
}

ts::VerifyKernelInfo ts::verify_kernel_info(int id)
{
    switch (id) {
        case kNarrow_16: return {16, 5};
        case kNarrow_32: return {32, 4};
        case kWide_1x1: return {32, 3};
        case kWide_1x1b: return {32, 2};
        case kWide_1x2: case kWide_1x2h: return {64, 2};
        case kWide_1x2k4: return {64, 1};
        case kWide_1x4: case kWide_1x4h: return {128, 2};
        case kWide_1x4k3: case kWide_1x4k2h: return {128, 1};
        case kWide_2x4: case kWide_1x8: case kWide_1x8h: case kWide_1x8h4: return {256, 1};
        case kWide_1x10: case kWide_1x10h: return {320, 1};
        case kWide_1x12: case kWide_1x12h: return {384, 1};
        case kWide_2x2: return {128, 2};
        case kWide_2x2k2: case kWide_2x2k2b: return {128, 1};
        default: return {0, 0};
    }
}

extern "C" {

const char *ts_strerror(int status)
{
    switch (status) {
        case TS_OK: return "ok";
        case TS_ERR_NULL: return "a required pointer is NULL";
        case TS_ERR_SHAPE: return "sizes are inconsistent or out of range";
        case TS_ERR_UNSUPPORTED: return "shape not supported by the kernels";
        case TS_ERR_TREE: return "parent array is not a forest in topological order";
        case TS_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case TS_ERR_HIP: return "HIP runtime error";
        case TS_ERR_ALIGN: return "pointer or stride breaks 16-byte row alignment";
        default: return "unknown status";
    }
}

int ts_version(void) { return 210; }

int ts_tune_set(const char *name, int value)
{
    if (!name || value < 0) return TS_ERR_UNSUPPORTED;
    if (strcmp(name, "verify_splits") == 0) {
        g_tune.verify_splits = value;
        return TS_OK;
    }
    if (strcmp(name, "verify_kernel") == 0) {
        if (value > ts::kVerifyKernelCount) return TS_ERR_UNSUPPORTED;
        g_tune.verify_kernel = value;
        return TS_OK;
    }
    if (strcmp(name, "verify_variant") == 0) {
        if (value > 3) return TS_ERR_UNSUPPORTED;
        g_tune.verify_variant = value;
        return TS_OK;
    }
    return TS_ERR_UNSUPPORTED;
}

size_t ts_workspace_bytes(int op, int n_q_heads, int n_kv_heads, int64_t n_tokens, int n_tree,
                          int n_sel, int chunk_size)
{
    int group = 0;
    if (check_heads(n_q_heads, n_kv_heads, &group) != TS_OK) return 0;
    if (op == TS_OP_TREE_VERIFY || op == TS_OP_TREE_VERIFY_SCORED) {
        if (n_tree < 1 || n_tree > TS_MAX_TREE || n_tokens < 0) return 0;
        VerifyPlan pl;
        if (!plan_verify(n_q_heads, n_kv_heads, n_tokens, n_tree, op == TS_OP_TREE_VERIFY_SCORED, &pl)) return 0;
        return pl.bytes;
    }
    if (op == TS_OP_PARTIAL_ATTN) {
        if (n_sel < 1 || n_sel > TS_MAX_CHUNKS || !partial_chunk_ok(chunk_size)) return 0;
        PartialPlan pl;
        plan_partial(n_q_heads, n_kv_heads, n_sel, chunk_size, &pl);
        return pl.bytes;
    }
    return 0;
}

int ts_chunk_scores(const ts_kv_view *kv, const void *q, int n_q_heads, int chunk_size,
                    float scale, float *scores, void *stream)
{
    int rc = check_view(kv, false, false);
    if (rc != TS_OK) return rc;
    if (!q || !scores) return TS_ERR_NULL;
    int group = 0;
    if ((rc = check_heads(n_q_heads, kv->n_kv_heads, &group)) != TS_OK) return rc;
    if (chunk_size < 1 || chunk_size > 1024) return TS_ERR_UNSUPPORTED;
    if (!aligned16(q)) return TS_ERR_ALIGN;
    ts::ScoresParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.k = static_cast<const uint16_t *>(kv->k);
    p.scores = scores;
    p.stride_head = kv->stride_head;
    p.stride_token = kv->stride_token;
    p.n_tokens = kv->n_tokens;
    p.n_chunks = (kv->n_tokens + chunk_size - 1) / chunk_size;
    if ((p.n_chunks + 3) / 4 > 0x7fffffffLL) return TS_ERR_UNSUPPORTED;
    p.n_q_heads = n_q_heads;
    p.n_kv_heads = kv->n_kv_heads;
    p.group = group;
    p.chunk_size = chunk_size;
    p.scale = scale;
    return ts::launch_scores(p, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_topk_chunks(const float *scores, int n_kv_heads, int n_chunks, int n_sink_chunks, int k,
                   int32_t *idx_out, void *stream)
{
    if (!scores || !idx_out) return TS_ERR_NULL;
    if (n_kv_heads < 1 || n_chunks < 1 || n_sink_chunks < 0 || k < 0) return TS_ERR_SHAPE;
    if ((int64_t)n_sink_chunks + k > n_chunks || n_sink_chunks + k < 1) return TS_ERR_SHAPE;
    if (n_chunks > TS_MAX_CHUNKS || k > TS_MAX_TOPK) return TS_ERR_UNSUPPORTED;
    ts::TopkParams p;
    p.scores = scores;
    p.idx_out = idx_out;
    p.n_kv_heads = n_kv_heads;
    p.n_chunks = n_chunks;
    p.n_sink = n_sink_chunks;
    p.k = k;
    return ts::launch_topk(p, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_partial_kv_attn(const ts_kv_view *kv, const void *q, int n_q_heads,
                       const int32_t *chunk_idx, int n_sel, int chunk_size, float scale,
                       float *out, float *lse, void *workspace, size_t workspace_bytes,
                       void *stream)
{
    int rc = check_view(kv, true, false);
    if (rc != TS_OK) return rc;
    if (!q || !chunk_idx || !out) return TS_ERR_NULL;
    int group = 0;
    if ((rc = check_heads(n_q_heads, kv->n_kv_heads, &group)) != TS_OK) return rc;
    if (n_sel < 1) return TS_ERR_SHAPE;
    if (n_sel > TS_MAX_CHUNKS || !partial_chunk_ok(chunk_size) || !scale_ok(scale)) return TS_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(out)) return TS_ERR_ALIGN;
    PartialPlan pl;
    plan_partial(n_q_heads, kv->n_kv_heads, n_sel, chunk_size, &pl);
    if (!workspace || workspace_bytes < pl.bytes || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return TS_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    ts::PartialParams p;
    p.q = static_cast<const uint16_t *>(q);
    p.k = static_cast<const uint16_t *>(kv->k);
    p.v = static_cast<const uint16_t *>(kv->v);
    p.chunk_idx = chunk_idx;
    p.ws_o = reinterpret_cast<float *>(workspace);
    p.ws_ml = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + pl.ml_offset);
    p.stride_head = kv->stride_head;
    p.stride_token = kv->stride_token;
    p.n_tokens = kv->n_tokens;
    p.n_q_heads = n_q_heads;
    p.n_kv_heads = kv->n_kv_heads;
    p.group = group;
    p.n_sel = n_sel;
    p.chunk_size = chunk_size;
    p.segs_per_chunk = pl.segs_per_chunk;
    p.n_seg = pl.n_seg;
    p.n_part = pl.n_part;
    p.scale_log2 = scale * 1.4426950408889634f;
    if (ts::launch_partial(p, st) != hipSuccess) return TS_ERR_HIP;

    ts::CombineParams c{};
    c.ws_o = p.ws_o;
    c.ws_ml = p.ws_ml;
    c.out = out;
    c.lse = lse;
    c.n_kv_heads = kv->n_kv_heads;
    c.n_q_heads = n_q_heads;
    c.group = group;
    c.n_part = pl.n_part;
    c.n_rows = group;
    c.row_pitch = group;
    return ts::launch_combine(c, st) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_partial_kv_attn_static(const ts_kv_view *kv, const void *q, int n_q_heads,
                              const int32_t *chunk_idx, int n_sel, int chunk_size, float scale,
                              float *out, float *lse, void *stream)
{
    // same validation as ts_partial_kv_attn up to the workspace (repeated here so that a shape error is not
    // reported as a size error), then the size limit, then the same launches with the static array
    int rc = check_view(kv, true, false);
    if (rc != TS_OK) return rc;
    if (!q || !chunk_idx || !out) return TS_ERR_NULL;
    int group = 0;
    if ((rc = check_heads(n_q_heads, kv->n_kv_heads, &group)) != TS_OK) return rc;
    if (n_sel < 1) return TS_ERR_SHAPE;
    if (n_sel > TS_MAX_CHUNKS || !partial_chunk_ok(chunk_size) || !scale_ok(scale)) return TS_ERR_UNSUPPORTED;
    PartialPlan pl;
    plan_partial(n_q_heads, kv->n_kv_heads, n_sel, chunk_size, &pl);
    if (pl.bytes > kScratchBytes) return TS_ERR_WORKSPACE;    // beyond the fixed scratch: use ts_partial_kv_attn
    void *ptr = nullptr;
    if ((rc = scratch_of_current_device(&ptr)) != TS_OK) return rc;
    return ts_partial_kv_attn(kv, q, n_q_heads, chunk_idx, n_sel, chunk_size, scale, out, lse, ptr, kScratchBytes, stream);
}

// ts_tree_verify_attn, and with scores != nullptr ts_tree_verify_attn_scored
// split_only: enqueue the split kernel alone (ts_bench_verify_split_kernel); out is then unused
static int verify_call(const ts_kv_view *kv, const void *q_tree, int n_q_heads,
                       const void *k_tree, const void *v_tree, const int32_t *parent,
                       int n_tree, float scale, int chunk_size, float *scores, float *out, float *lse,
                       void *workspace, size_t workspace_bytes, void *stream, bool split_only = false, bool split_only_sums = false)
{
    const bool scored = scores != nullptr || split_only_sums;   // the split kernel also leaves the per-tile logit sums
    int rc = check_view(kv, true, true);
    if (rc != TS_OK) return rc;
    if (!q_tree || !k_tree || !v_tree || !parent || (!out && !split_only)) return TS_ERR_NULL;
    int group = 0;
    if ((rc = check_heads(n_q_heads, kv->n_kv_heads, &group)) != TS_OK) return rc;
    if (n_tree < 1) return TS_ERR_SHAPE;
    if (n_tree > TS_MAX_TREE || !scale_ok(scale)) return TS_ERR_UNSUPPORTED;
    if (kv->n_tokens > 0x7fffffffLL) return TS_ERR_UNSUPPORTED;   // the kernels keep positions inside a range in 32 bits
    for (int i = 0; i < n_tree; ++i)
        if (parent[i] < -1 || parent[i] >= i) return TS_ERR_TREE;
    if (!aligned16(q_tree) || !aligned16(k_tree) || !aligned16(v_tree) || (out && !aligned16(out))) return TS_ERR_ALIGN;
    VerifyPlan pl;
    if (!plan_verify(n_q_heads, kv->n_kv_heads, kv->n_tokens, n_tree, scored, &pl)) return TS_ERR_UNSUPPORTED;
    if (!workspace || workspace_bytes < pl.bytes || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return TS_ERR_WORKSPACE;

    hipStream_t st = static_cast<hipStream_t>(stream);
    ts::VerifyParams p;
    p.q = static_cast<const uint16_t *>(q_tree);
    p.k = static_cast<const uint16_t *>(kv->k);
    p.v = static_cast<const uint16_t *>(kv->v);
    p.k_tree = static_cast<const uint16_t *>(k_tree);
    p.v_tree = static_cast<const uint16_t *>(v_tree);
    p.ws_o = reinterpret_cast<float *>(workspace);
    p.ws_ml = reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + pl.ml_offset);
    p.tile_sums = scored ? reinterpret_cast<float *>(static_cast<unsigned char *>(workspace) + pl.tile_offset) : nullptr;
    p.tile_sums_stride = pl.n_tiles;
    p.stride_head = kv->stride_head;
    p.stride_token = kv->stride_token;
    p.n_tokens = kv->n_tokens;
    p.split_len = pl.split_len;
    p.n_split = pl.n_split;
    p.n_q_heads = n_q_heads;
    p.n_kv_heads = kv->n_kv_heads;
    p.group = group;
    p.n_tree = n_tree;
    p.n_rows = pl.n_rows;
    p.n_rows_pad = pl.n_rows_pad;
    p.rows_per_wg = pl.shape.rows_per_wg;
    p.scale_log2 = scale * 1.4426950408889634f;
    // ancestor-or-self bit masks (App. E: a node attends only to its predecessors)
    memset(p.anc, 0, sizeof(p.anc));
    for (int i = 0; i < n_tree; ++i) {
        if (parent[i] >= 0) {
            p.anc[i][0] = p.anc[parent[i]][0];
            p.anc[i][1] = p.anc[parent[i]][1];
        }
        p.anc[i][i >> 6] |= 1ull << (i & 63);
    }
    {
        const hipError_t e = pl.shape.kernel_id <= ts::kNarrow_32 ? ts::launch_verify_narrow(p, pl.shape.kernel_id, st)
                                                                  : ts::launch_verify_wide(p, pl.shape.kernel_id, st);
        if (e != hipSuccess) return TS_ERR_HIP;
    }
    if (split_only) return TS_OK;

    ts::CombineParams c{};
    c.ws_o = p.ws_o;
    c.ws_ml = p.ws_ml;
    c.out = out;
    c.lse = lse;
    c.n_kv_heads = kv->n_kv_heads;
    c.n_q_heads = n_q_heads;
    c.group = group;
    c.n_part = pl.n_split + 1;
    c.n_rows = pl.n_rows;
    c.row_pitch = pl.n_rows_pad;
    c.tile_sums = p.tile_sums;
    c.scores = scores;
    c.tile_sums_stride = pl.n_tiles;
    c.n_tokens = kv->n_tokens;
    c.chunk_size = chunk_size;
    c.n_chunks = scores ? (kv->n_tokens + chunk_size - 1) / chunk_size : 0;
    c.scale = scale;
    return ts::launch_combine(c, st) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_tree_verify_attn(const ts_kv_view *kv, const void *q_tree, int n_q_heads,
                        const void *k_tree, const void *v_tree, const int32_t *parent,
                        int n_tree, float scale, float *out, float *lse, void *workspace,
                        size_t workspace_bytes, void *stream)
{
    return verify_call(kv, q_tree, n_q_heads, k_tree, v_tree, parent, n_tree, scale, 0, nullptr, out, lse, workspace,
                       workspace_bytes, stream);
}

int ts_tree_verify_attn_scored(const ts_kv_view *kv, const void *q_tree, int n_q_heads,
                               const void *k_tree, const void *v_tree, const int32_t *parent,
                               int n_tree, float scale, int chunk_size, float *scores, float *out,
                               float *lse, void *workspace, size_t workspace_bytes, void *stream)
{
    if (!scores) return TS_ERR_NULL;
    if (kv && kv->n_tokens < 1) return TS_ERR_SHAPE;                         // nothing to score
    if (chunk_size < 32 || chunk_size > 1024 || chunk_size % 32 != 0) return TS_ERR_UNSUPPORTED;   // whole 32-key tiles
    return verify_call(kv, q_tree, n_q_heads, k_tree, v_tree, parent, n_tree, scale, chunk_size, scores, out, lse, workspace,
                       workspace_bytes, stream);
}

int ts_bench_verify_split_kernel(const ts_kv_view *kv, const void *q_tree, int n_q_heads,
                                 const void *k_tree, const void *v_tree, const int32_t *parent,
                                 int n_tree, float scale, int with_tile_sums, void *workspace,
                                 size_t workspace_bytes, void *stream)
{
    if (with_tile_sums && kv && kv->n_tokens < 1) return TS_ERR_SHAPE;
    return verify_call(kv, q_tree, n_q_heads, k_tree, v_tree, parent, n_tree, scale, 32, nullptr, nullptr, nullptr, workspace,
                       workspace_bytes, stream, true, with_tile_sums != 0);
}

int ts_append_accepted(const ts_kv_view *kv, const void *k_tree, const void *v_tree, int n_tree,
                       const int32_t *accepted, int n_accepted, void *stream)
{
    if (!kv) return TS_ERR_NULL;
    if (kv->head_dim != TS_HEAD_DIM) return TS_ERR_UNSUPPORTED;
    if (kv->n_kv_heads < 1 || kv->n_tokens < 0) return TS_ERR_SHAPE;
    if (kv->n_kv_heads > 65535) return TS_ERR_UNSUPPORTED;
    if (!kv->k || !kv->v || !k_tree || !v_tree || !accepted) return TS_ERR_NULL;
    if (kv->stride_token < TS_HEAD_DIM || kv->stride_head < 0) return TS_ERR_SHAPE;
    if ((kv->stride_token % 8) != 0 || (kv->stride_head % 8) != 0) return TS_ERR_ALIGN;
    if (!aligned16(kv->k) || !aligned16(kv->v) || !aligned16(k_tree) || !aligned16(v_tree)) return TS_ERR_ALIGN;
    if (n_tree < 1 || n_accepted < 1) return TS_ERR_SHAPE;
    if (n_tree > TS_MAX_TREE || n_accepted > TS_MAX_TREE) return TS_ERR_UNSUPPORTED;
    ts::AppendParams p;
    for (int i = 0; i < n_accepted; ++i) {
        if (accepted[i] < 0 || accepted[i] >= n_tree) return TS_ERR_TREE;
        p.accepted[i] = accepted[i];
    }
    for (int i = n_accepted; i < ts::kMaxTree; ++i) p.accepted[i] = 0;
    p.k = static_cast<uint16_t *>(const_cast<void *>(kv->k));
    p.v = static_cast<uint16_t *>(const_cast<void *>(kv->v));
    p.k_tree = static_cast<const uint16_t *>(k_tree);
    p.v_tree = static_cast<const uint16_t *>(v_tree);
    p.stride_head = kv->stride_head;
    p.stride_token = kv->stride_token;
    p.n_tokens = kv->n_tokens;
    p.n_kv_heads = kv->n_kv_heads;
    p.n_accepted = n_accepted;
    return ts::launch_append(p, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_refresh_due(int64_t n_tokens, int64_t n_tokens_at_refresh, int64_t budget_tokens, int64_t sink_tokens)
{
    if (n_tokens < 0 || n_tokens_at_refresh < 0 || n_tokens_at_refresh > n_tokens || sink_tokens < 0 ||
        budget_tokens < sink_tokens)
        return TS_ERR_SHAPE;
    return (n_tokens - n_tokens_at_refresh) > (budget_tokens - sink_tokens) ? 1 : 0;
}

int ts_chunk_list_admit(int32_t *chunk_idx, int n_kv_heads, int n_sel, int n_sink_chunks, int base_chunk,
                        int first_new_chunk, int n_new_chunks, void *stream)
{
    if (!chunk_idx) return TS_ERR_NULL;
    if (n_kv_heads < 1 || n_sel < 1 || n_sink_chunks < 0 || n_sink_chunks > n_sel || base_chunk < 0) return TS_ERR_SHAPE;
    if (n_kv_heads > 65535) return TS_ERR_UNSUPPORTED;
    if (n_new_chunks < 0 || first_new_chunk < base_chunk) return TS_ERR_SHAPE;
    if ((int64_t)first_new_chunk + n_new_chunks > 0x7fffffffLL) return TS_ERR_SHAPE;
    if ((int64_t)first_new_chunk + n_new_chunks - base_chunk > n_sel - n_sink_chunks) return TS_ERR_SHAPE;   // a rebuild is due instead
    if (n_new_chunks == 0) return TS_OK;
    return ts::launch_admit(chunk_idx, n_kv_heads, n_sel, n_sink_chunks, base_chunk, first_new_chunk, n_new_chunks,
                            static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_gather_chunks(const ts_kv_view *kv, const int32_t *chunk_idx, int n_sel, int chunk_size,
                     void *k_out, void *v_out, void *stream)
{
    int rc = check_view(kv, true, false);
    if (rc != TS_OK) return rc;
    if (!chunk_idx || !k_out || !v_out) return TS_ERR_NULL;
    if (n_sel < 1) return TS_ERR_SHAPE;
    if (n_sel > TS_MAX_CHUNKS || !partial_chunk_ok(chunk_size)) return TS_ERR_UNSUPPORTED;
    if (!aligned16(k_out) || !aligned16(v_out)) return TS_ERR_ALIGN;
    if ((int64_t)n_sel * chunk_size / 16 > 0x7fffffffLL) return TS_ERR_UNSUPPORTED;
    ts::GatherParams p;
    p.k = static_cast<const uint16_t *>(kv->k);
    p.v = static_cast<const uint16_t *>(kv->v);
    p.chunk_idx = chunk_idx;
    p.k_out = static_cast<uint16_t *>(k_out);
    p.v_out = static_cast<uint16_t *>(v_out);
    p.stride_head = kv->stride_head;
    p.stride_token = kv->stride_token;
    p.n_tokens = kv->n_tokens;
    p.n_kv_heads = kv->n_kv_heads;
    p.n_sel = n_sel;
    p.chunk_size = chunk_size;
    return ts::launch_gather(p, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_chunk_key_sums(const ts_kv_view *kv, int chunk_size, int64_t chunk_begin, int64_t chunk_end,
                      float *ksum, int64_t ksum_stride_head, void *stream)
{
    int rc = check_view(kv, false, false);
    if (rc != TS_OK) return rc;
    if (!ksum) return TS_ERR_NULL;
    if (chunk_size < 1 || chunk_size > 1024) return TS_ERR_UNSUPPORTED;
    const int64_t n_chunks = (kv->n_tokens + chunk_size - 1) / chunk_size;
    if (chunk_begin < 0 || chunk_end < chunk_begin || chunk_end > n_chunks) return TS_ERR_SHAPE;
    if (ksum_stride_head < n_chunks * TS_HEAD_DIM && kv->n_kv_heads > 1) return TS_ERR_SHAPE;
    if (!aligned16(ksum) || (ksum_stride_head % 4) != 0) return TS_ERR_ALIGN;
    if (chunk_end == chunk_begin) return TS_OK;
    if ((chunk_end - chunk_begin + 3) / 4 > 0x7fffffffLL) return TS_ERR_UNSUPPORTED;
    ts::KsumParams p;
    p.k = static_cast<const uint16_t *>(kv->k);
    p.ksum = ksum;
    p.stride_head = kv->stride_head;
    p.stride_token = kv->stride_token;
    p.ksum_stride_head = ksum_stride_head;
    p.n_tokens = kv->n_tokens;
    p.chunk_begin = chunk_begin;
    p.chunk_end = chunk_end;
    p.n_kv_heads = kv->n_kv_heads;
    p.chunk_size = chunk_size;
    return ts::launch_ksum(p, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_chunk_scores_from_sums(const float *ksum, int64_t ksum_stride_head, int n_kv_heads,
                              int64_t n_tokens, const void *q, int n_q_heads, int chunk_size,
                              float scale, float *scores, void *stream)
{
    if (!ksum || !q || !scores) return TS_ERR_NULL;
    int group = 0;
    int rc = check_heads(n_q_heads, n_kv_heads, &group);
    if (rc != TS_OK) return rc;
    if (n_tokens < 1) return TS_ERR_SHAPE;
    if (chunk_size < 1 || chunk_size > 1024) return TS_ERR_UNSUPPORTED;
    const int64_t n_chunks = (n_tokens + chunk_size - 1) / chunk_size;
    if (ksum_stride_head < n_chunks * TS_HEAD_DIM && n_kv_heads > 1) return TS_ERR_SHAPE;
    if (!aligned16(ksum) || (ksum_stride_head % 4) != 0 || !aligned16(q)) return TS_ERR_ALIGN;
    if ((n_chunks + 3) / 4 > 0x7fffffffLL) return TS_ERR_UNSUPPORTED;
    ts::SumScoresParams p;
    p.ksum = ksum;
    p.q = static_cast<const uint16_t *>(q);
    p.scores = scores;
    p.ksum_stride_head = ksum_stride_head;
    p.n_tokens = n_tokens;
    p.n_chunks = n_chunks;
    p.n_kv_heads = n_kv_heads;
    p.group = group;
    p.chunk_size = chunk_size;
    p.scale = scale;
    return ts::launch_sum_scores(p, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

size_t ts_sampling_workspace_bytes(int n_rows, int64_t vocab)
{
    if (n_rows < 1 || vocab < 1 || vocab > (1 << 24)) return 0;
    return round_up((size_t)n_rows * ts::sampling_slices(vocab) * 2 * sizeof(float), 256);
}

int ts_penalized_probs(const float *logits, int n_rows, int64_t vocab, const int32_t *window,
                       int n_window, float temperature, float theta, float *probs, void *workspace,
                       size_t workspace_bytes, void *stream)
{
    if (!logits || !probs || (n_window > 0 && !window)) return TS_ERR_NULL;
    if (n_rows < 1 || vocab < 1 || n_window < 0) return TS_ERR_SHAPE;
    if (vocab > (1 << 24) || n_rows > 65535) return TS_ERR_UNSUPPORTED;
    if (!(temperature > 0.f && temperature < 3.0e38f) || !(theta >= 1.f && theta < 3.0e38f)) return TS_ERR_UNSUPPORTED;
    if (!aligned16(logits) || !aligned16(probs)) return TS_ERR_ALIGN;
    const size_t need = ts_sampling_workspace_bytes(n_rows, vocab);
    if (!workspace || workspace_bytes < need || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return TS_ERR_WORKSPACE;
    ts::PenaltyParams p;
    p.logits = logits;
    p.probs = probs;
    p.window = window;
    p.n_window = n_window;
    p.stats = static_cast<float *>(workspace);
    p.vocab = vocab;
    p.n_rows = n_rows;
    p.n_slices = ts::sampling_slices(vocab);
    p.k_plain = 1.4426950408889634f / temperature;
    p.k_window = 1.4426950408889634f / (temperature * theta);
    return ts::launch_penalized_probs(p, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_sample_tokens(const float *probs, int n_rows, int64_t vocab, int method, float param,
                     float param2, const float *u, int32_t *tokens, float *pool_threshold,
                     float *pool_mass, void *stream)
{
    if (!probs || !u || !tokens) return TS_ERR_NULL;
    if (n_rows < 1 || vocab < 1) return TS_ERR_SHAPE;
    if (vocab > (1 << 24)) return TS_ERR_UNSUPPORTED;
    if (method < TS_SAMPLE_FULL || method > TS_SAMPLE_ETA) return TS_ERR_UNSUPPORTED;
    if (method == TS_SAMPLE_ETA && !(param2 > 0.f && param2 < 3.0e38f)) return TS_ERR_UNSUPPORTED;
    if (method != TS_SAMPLE_FULL && !(param > 0.f && param <= 1.f)) return TS_ERR_UNSUPPORTED;
    ts::SampleParams p;
    p.probs = probs;
    p.u = u;
    p.tokens = tokens;
    p.pool_threshold = pool_threshold;
    p.pool_mass = pool_mass;
    p.vocab = vocab;
    p.n_rows = n_rows;
    p.method = method;
    p.param = param;
    p.param2 = param2;
    return ts::launch_sample(p, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

int ts_stream_read_probe(const void *src, size_t bytes, uint32_t *sink, void *stream)
{
    if (!src || !sink) return TS_ERR_NULL;
    if (bytes < 16 || bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(src) & 15u) != 0) return TS_ERR_SHAPE;
    if (bytes / 16 / 2048 >= 0x7fffffffULL) return TS_ERR_UNSUPPORTED;
    return ts::launch_stream_read(src, (int64_t)(bytes / 16), sink, static_cast<hipStream_t>(stream)) == hipSuccess ? TS_OK : TS_ERR_HIP;
}

}  // extern "C"
