"""MI355X-native decode-attention hot path of TokenSwift (arXiv 2502.18890).

Thin Python front end of ``libtokenswift_hip.so`` (C ABI in ``include/tokenswift.h``): chunk
importance scores, top-k chunk selection, partial-KV attention and tree-verification attention
as hand-written gfx950 kernels.  PyTorch is used only for device memory and streams.
"""
from .binding import (TokenSwiftError, append_accepted, bench_verify_split_kernel, chunk_key_sums, chunk_list_admit, chunk_scores,
                      chunk_scores_from_sums, gather_chunks, lib_path, load_library, partial_kv_attn, partial_kv_attn_static,
                      penalized_probs, refresh_due, sample_tokens, stream_read_probe, topk_chunks, tree_verify_attn, tune_set, version, workspace_bytes,
                      OP_PARTIAL_ATTN, OP_TREE_VERIFY, OP_TREE_VERIFY_SCORED, SAMPLE_ETA, SAMPLE_FULL, SAMPLE_MIN_P, SAMPLE_TOP_P)

__all__ = ["TokenSwiftError", "append_accepted", "bench_verify_split_kernel", "chunk_key_sums", "chunk_list_admit", "chunk_scores_from_sums",
           "gather_chunks", "penalized_probs", "refresh_due", "sample_tokens", "chunk_scores", "lib_path", "load_library", "partial_kv_attn", "partial_kv_attn_static",
           "stream_read_probe", "topk_chunks", "tree_verify_attn", "tune_set", "version", "workspace_bytes",
           "OP_PARTIAL_ATTN", "OP_TREE_VERIFY", "OP_TREE_VERIFY_SCORED", "SAMPLE_ETA", "SAMPLE_FULL", "SAMPLE_MIN_P", "SAMPLE_TOP_P"]
