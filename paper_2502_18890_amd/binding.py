"""ctypes binding of the C ABI declared in include/tokenswift.h.

Argument marshalling only: every step of the path runs in the HIP kernels.  There is no
fallback: if the shared library is missing the import of the first function fails loudly.
Tensors are torch tensors on the GPU (bf16 for q/K/V, fp32/int32 for the rest); ``parent`` is a
host sequence.  Work is enqueued on torch's current stream.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("TOKENSWIFT_LIB", os.path.join(_PKG, "libtokenswift_hip.so"))   # override: another build of the same ABI

OP_PARTIAL_ATTN = 1
OP_TREE_VERIFY = 2
OP_TREE_VERIFY_SCORED = 3
HEAD_DIM = 128


class TokenSwiftError(RuntimeError):
    def __init__(self, status: int, text: str, where: str):
        super().__init__("%s: %s (status %d)" % (where, text, status))
        self.status = status


class _KvView(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("n_tokens", ctypes.c_int64),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("stride_head", ctypes.c_int64), ("stride_token", ctypes.c_int64)]


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libtokenswift_hip.so (built by paper_2502_18890_amd.build); raises if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError("%s not found: build it with `python -m paper_2502_18890_amd.build` "
                          "(there is no CPU fallback)" % _LIB_PATH)
    lib = ctypes.CDLL(_LIB_PATH)
    vp, ci, i64, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_float
    kvp = ctypes.POINTER(_KvView)
    lib.ts_strerror.argtypes = [ci]
    lib.ts_strerror.restype = ctypes.c_char_p
    lib.ts_version.restype = ci
    lib.ts_tune_set.argtypes = [ctypes.c_char_p, ci]
    lib.ts_workspace_bytes.argtypes = [ci, ci, ci, i64, ci, ci, ci]
    lib.ts_workspace_bytes.restype = ctypes.c_size_t
    lib.ts_chunk_scores.argtypes = [kvp, vp, ci, ci, cf, vp, vp]
    lib.ts_topk_chunks.argtypes = [vp, ci, ci, ci, ci, vp, vp]
    lib.ts_partial_kv_attn.argtypes = [kvp, vp, ci, vp, ci, ci, cf, vp, vp, vp, ctypes.c_size_t, vp]
    lib.ts_partial_kv_attn_static.argtypes = [kvp, vp, ci, vp, ci, ci, cf, vp, vp, vp]
    lib.ts_partial_kv_attn_static.restype = ci
    lib.ts_tree_verify_attn.argtypes = [kvp, vp, ci, vp, vp, ctypes.POINTER(ctypes.c_int32), ci, cf,
                                        vp, vp, vp, ctypes.c_size_t, vp]
    lib.ts_tree_verify_attn_scored.argtypes = [kvp, vp, ci, vp, vp, ctypes.POINTER(ctypes.c_int32), ci, cf, ci, vp,
                                               vp, vp, vp, ctypes.c_size_t, vp]
    i32p = ctypes.POINTER(ctypes.c_int32)
    lib.ts_bench_verify_split_kernel.argtypes = [kvp, vp, ci, vp, vp, i32p, ci, cf, ci, vp, ctypes.c_size_t, vp]
    lib.ts_append_accepted.argtypes = [kvp, vp, vp, ci, i32p, ci, vp]
    lib.ts_refresh_due.argtypes = [i64, i64, i64, i64]
    lib.ts_chunk_list_admit.argtypes = [vp, ci, ci, ci, ci, ci, ci, vp]
    lib.ts_gather_chunks.argtypes = [kvp, vp, ci, ci, vp, vp, vp]
    lib.ts_chunk_key_sums.argtypes = [kvp, ci, i64, i64, vp, i64, vp]
    lib.ts_chunk_scores_from_sums.argtypes = [vp, i64, ci, i64, vp, ci, ci, cf, vp, vp]
    lib.ts_sampling_workspace_bytes.argtypes = [ci, i64]
    lib.ts_sampling_workspace_bytes.restype = ctypes.c_size_t
    lib.ts_penalized_probs.argtypes = [vp, ci, i64, vp, ci, cf, cf, vp, vp, ctypes.c_size_t, vp]
    lib.ts_sample_tokens.argtypes = [vp, ci, i64, ci, cf, cf, vp, vp, vp, vp, vp]
    lib.ts_penalized_probs.restype = ci
    lib.ts_sample_tokens.restype = ci
    lib.ts_stream_read_probe.argtypes = [vp, ctypes.c_size_t, vp, vp]
    for name in ("ts_bench_verify_split_kernel", "ts_stream_read_probe", "ts_tune_set", "ts_chunk_scores", "ts_topk_chunks", "ts_partial_kv_attn",
                 "ts_tree_verify_attn", "ts_tree_verify_attn_scored", "ts_append_accepted", "ts_refresh_due", "ts_chunk_list_admit",
                 "ts_gather_chunks", "ts_chunk_key_sums", "ts_chunk_scores_from_sums"):
        getattr(lib, name).restype = ci
    _lib = lib
    return lib


def _check(status: int, where: str) -> None:
    if status != 0:
        raise TokenSwiftError(status, load_library().ts_strerror(status).decode(), where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _view(k: Optional[torch.Tensor], v: Optional[torch.Tensor], n_kv_heads: Optional[int] = None) -> _KvView:
    """k, v: [n_kv_heads, n_tokens, 128] bf16 views (any head/token strides, unit stride in d)."""
    if k is None:
        return _KvView(None, None, 0, int(n_kv_heads), HEAD_DIM, 0, HEAD_DIM)
    if k.dtype != torch.bfloat16 or k.dim() != 3 or k.stride(2) != 1:
        raise ValueError("cache must be a bf16 [n_kv_heads, n_tokens, d] view with unit stride in d")
    if v is not None and (v.dtype != k.dtype or v.shape != k.shape or v.stride() != k.stride()):
        raise ValueError("v must match k in dtype, shape and strides")
    return _KvView(k.data_ptr(), v.data_ptr() if v is not None else None, k.shape[1], k.shape[0],
                   k.shape[2], k.stride(0), k.stride(1))


def version() -> int:
    return int(load_library().ts_version())


def tune_set(name: str, value: int) -> None:
    _check(load_library().ts_tune_set(name.encode(), int(value)), "ts_tune_set")


def stream_read_probe(buf: torch.Tensor, sink: torch.Tensor) -> None:
    """Reads the contiguous tensor `buf` once (measurement utility); `sink`: a 4-byte device tensor."""
    if not buf.is_contiguous():
        raise ValueError("buf must be contiguous")
    _check(load_library().ts_stream_read_probe(buf.data_ptr(), buf.numel() * buf.element_size(), sink.data_ptr(), _stream()),
           "ts_stream_read_probe")


def workspace_bytes(op: int, n_q_heads: int, n_kv_heads: int, n_tokens: int, n_tree: int = 0,
                    n_sel: int = 0, chunk_size: int = 0) -> int:
    return int(load_library().ts_workspace_bytes(op, n_q_heads, n_kv_heads, n_tokens, n_tree, n_sel,
                                                 chunk_size))


def _workspace(nbytes: int, device, workspace: Optional[torch.Tensor]) -> torch.Tensor:
    if nbytes == 0:
        raise ValueError("shape rejected by ts_workspace_bytes")
    if workspace is None:
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return workspace


_parent_cache: dict = {}


def _parent_array(parent: Sequence[int]):
    """Host int32 array of the tree for the C call; the same tree is usually passed call after call."""
    key = (len(parent), str(parent.dtype), parent.tobytes()) if hasattr(parent, "tobytes") else tuple(int(x) for x in parent)
    arr = _parent_cache.get(key)
    if arr is None:
        if len(_parent_cache) > 256:
            _parent_cache.clear()
        arr = (ctypes.c_int32 * len(parent))(*[int(x) for x in parent])
        _parent_cache[key] = arr
    return arr


def chunk_scores(q: torch.Tensor, k: torch.Tensor, chunk_size: int, scale: float,
                 out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """q [Hq,128] bf16, k [Hkv,N,128] bf16 view -> scores fp32 [Hkv, ceil(N/chunk_size)]."""
    lib = load_library()
    kv = _view(k, None)
    n_chunks = (k.shape[1] + chunk_size - 1) // chunk_size if chunk_size > 0 else 0
    if out is None:
        out = torch.empty(k.shape[0], max(n_chunks, 1), dtype=torch.float32, device=k.device)
    q = q.contiguous()
    _check(lib.ts_chunk_scores(ctypes.byref(kv), q.data_ptr(), q.shape[0], int(chunk_size), float(scale),
                               out.data_ptr(), _stream()), "ts_chunk_scores")
    return out


def topk_chunks(scores: torch.Tensor, n_sink_chunks: int, k: int,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """scores fp32 [Hkv, n_chunks] -> idx int32 [Hkv, n_sink_chunks + k]."""
    lib = load_library()
    scores = scores.contiguous()
    if out is None:
        out = torch.empty(scores.shape[0], max(n_sink_chunks + k, 1), dtype=torch.int32, device=scores.device)
    _check(lib.ts_topk_chunks(scores.data_ptr(), scores.shape[0], scores.shape[1], int(n_sink_chunks), int(k),
                              out.data_ptr(), _stream()), "ts_topk_chunks")
    return out


def partial_kv_attn(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, chunk_idx: torch.Tensor,
                    chunk_size: int, scale: float, out: Optional[torch.Tensor] = None,
                    lse: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None,
                    want_lse: bool = False):
    """q [Hq,128], k/v [Hkv,N,128] bf16 views, chunk_idx int32 [Hkv,n_sel] -> out fp32 [Hq,128]
    (and lse fp32 [Hq] when want_lse or lse is given)."""
    lib = load_library()
    kv = _view(k, v)
    q = q.contiguous()
    chunk_idx = chunk_idx.contiguous()
    hq = q.shape[0]
    if workspace is None:   # a caller's workspace is checked by the library itself
        workspace = _workspace(workspace_bytes(OP_PARTIAL_ATTN, hq, k.shape[0], k.shape[1], 0, chunk_idx.shape[1], chunk_size),
                               k.device, None)
    if out is None:
        out = torch.empty(hq, HEAD_DIM, dtype=torch.float32, device=k.device)
    if lse is None and want_lse:
        lse = torch.empty(hq, dtype=torch.float32, device=k.device)
    _check(lib.ts_partial_kv_attn(ctypes.byref(kv), q.data_ptr(), hq, chunk_idx.data_ptr(), chunk_idx.shape[1],
                                  int(chunk_size), float(scale), out.data_ptr(),
                                  lse.data_ptr() if lse is not None else None, workspace.data_ptr(),
                                  workspace.numel(), _stream()), "ts_partial_kv_attn")
    return (out, lse) if lse is not None else out


def partial_kv_attn_static(q: torch.Tensor, k: torch.Tensor, v: torch.Tensor, chunk_idx: torch.Tensor,
                           chunk_size: int, scale: float, out: torch.Tensor, lse: Optional[torch.Tensor] = None):
    """ts_partial_kv_attn_static: as partial_kv_attn, with the library's fixed scratch instead of a
    workspace.  Nothing is allocated here either: `out` (and `lse`) are the caller's, q and chunk_idx
    must already be contiguous."""
    if not q.is_contiguous() or not chunk_idx.is_contiguous():
        raise ValueError("q and chunk_idx must be contiguous")
    kv = _view(k, v)
    _check(load_library().ts_partial_kv_attn_static(ctypes.byref(kv), q.data_ptr(), q.shape[0], chunk_idx.data_ptr(),
                                                    chunk_idx.shape[1], int(chunk_size), float(scale), out.data_ptr(),
                                                    lse.data_ptr() if lse is not None else None, _stream()),
           "ts_partial_kv_attn_static")
    return (out, lse) if lse is not None else out


def tree_verify_attn(q_tree: torch.Tensor, k: Optional[torch.Tensor], v: Optional[torch.Tensor],
                     k_tree: torch.Tensor, v_tree: torch.Tensor, parent: Sequence[int], scale: float,
                     out: Optional[torch.Tensor] = None, lse: Optional[torch.Tensor] = None,
                     workspace: Optional[torch.Tensor] = None, want_lse: bool = False,
                     score_chunk: int = 0, scores: Optional[torch.Tensor] = None):
    """q_tree [T,Hq,128], k/v [Hkv,N,128] (or None for an empty cache), k_tree/v_tree [T,Hkv,128]
    bf16, parent host ints [T] -> out fp32 [T,Hq,128] (and lse fp32 [T,Hq]).
    With score_chunk > 0 the call is ts_tree_verify_attn_scored: the chunk scores of the cache for the
    query of tree node 0 (fp32 [Hkv, ceil(N/score_chunk)]) are written to `scores` (allocated if None)
    and returned last."""
    lib = load_library()
    q_tree = q_tree.contiguous()
    k_tree = k_tree.contiguous()
    v_tree = v_tree.contiguous()
    t, hq = q_tree.shape[0], q_tree.shape[1]
    hkv = k_tree.shape[1]
    kv = _view(k, v, hkv)
    n_tokens = 0 if k is None else k.shape[1]
    if len(parent) != t:
        raise ValueError("parent must have one entry per tree node")
    par = _parent_array(parent)
    scored = score_chunk > 0
    if workspace is None:   # a caller's workspace is checked by the library itself
        workspace = _workspace(workspace_bytes(OP_TREE_VERIFY_SCORED if scored else OP_TREE_VERIFY, hq, hkv, n_tokens, t),
                               q_tree.device, None)
    if out is None:
        out = torch.empty(t, hq, HEAD_DIM, dtype=torch.float32, device=q_tree.device)
    if lse is None and want_lse:
        lse = torch.empty(t, hq, dtype=torch.float32, device=q_tree.device)
    lse_ptr = lse.data_ptr() if lse is not None else None
    if scored:
        n_chunks = (n_tokens + score_chunk - 1) // score_chunk
        if scores is None:
            scores = torch.empty(hkv, max(n_chunks, 1), dtype=torch.float32, device=q_tree.device)
        elif scores.dtype != torch.float32 or not scores.is_contiguous() or scores.numel() < hkv * n_chunks:
            raise ValueError("scores must be a contiguous fp32 [Hkv, n_chunks] tensor")
        _check(lib.ts_tree_verify_attn_scored(ctypes.byref(kv), q_tree.data_ptr(), hq, k_tree.data_ptr(), v_tree.data_ptr(),
                                              par, t, float(scale), int(score_chunk), scores.data_ptr(), out.data_ptr(),
                                              lse_ptr, workspace.data_ptr(), workspace.numel(), _stream()),
               "ts_tree_verify_attn_scored")
        return (out, lse, scores) if lse is not None else (out, scores)
    _check(lib.ts_tree_verify_attn(ctypes.byref(kv), q_tree.data_ptr(), hq, k_tree.data_ptr(), v_tree.data_ptr(),
                                   par, t, float(scale), out.data_ptr(), lse_ptr, workspace.data_ptr(),
                                   workspace.numel(), _stream()), "ts_tree_verify_attn")
    return (out, lse) if lse is not None else out


def bench_verify_split_kernel(q_tree: torch.Tensor, k: torch.Tensor, v: torch.Tensor, k_tree: torch.Tensor,
                              v_tree: torch.Tensor, parent: Sequence[int], scale: float, workspace: torch.Tensor,
                              with_tile_sums: bool = False) -> None:
    """Measurement utility: enqueues only the cache-streaming kernel of the verification pass (no output)."""
    lib = load_library()
    t, hq = q_tree.shape[0], q_tree.shape[1]
    kv = _view(k, v, k_tree.shape[1])
    par = (ctypes.c_int32 * len(parent))(*[int(x) for x in parent])
    _check(lib.ts_bench_verify_split_kernel(ctypes.byref(kv), q_tree.data_ptr(), hq, k_tree.data_ptr(), v_tree.data_ptr(), par, t,
                                            float(scale), int(bool(with_tile_sums)), workspace.data_ptr(), workspace.numel(),
                                            _stream()), "ts_bench_verify_split_kernel")


# ---- cache maintenance -----------------------------------------------------------------------
def append_accepted(k: torch.Tensor, v: torch.Tensor, n_tokens: int, k_tree: torch.Tensor, v_tree: torch.Tensor,
                    accepted: Sequence[int]) -> int:
    """k/v [Hkv,cap,128] bf16 cache buffers holding n_tokens tokens; writes the accepted tree rows
    behind them (in place) and returns the new token count."""
    lib = load_library()
    if n_tokens + len(accepted) > k.shape[1]:
        raise ValueError("cache capacity exceeded")
    kv = _KvView(k.data_ptr(), v.data_ptr(), int(n_tokens), k.shape[0], k.shape[2], k.stride(0), k.stride(1))
    if k.stride(2) != 1 or v.stride() != k.stride():
        raise ValueError("K and V must share strides, innermost stride 1")
    k_tree, v_tree = k_tree.contiguous(), v_tree.contiguous()
    acc = (ctypes.c_int32 * len(accepted))(*[int(x) for x in accepted])
    _check(lib.ts_append_accepted(ctypes.byref(kv), k_tree.data_ptr(), v_tree.data_ptr(), k_tree.shape[0], acc,
                                  len(accepted), _stream()), "ts_append_accepted")
    return n_tokens + len(accepted)


def refresh_due(n_tokens: int, n_tokens_at_refresh: int, budget_tokens: int, sink_tokens: int) -> bool:
    rc = load_library().ts_refresh_due(int(n_tokens), int(n_tokens_at_refresh), int(budget_tokens), int(sink_tokens))
    if rc < 0:
        _check(rc, "ts_refresh_due")
    return bool(rc)


def chunk_list_admit(chunk_idx: torch.Tensor, n_sink_chunks: int, base_chunk: int, first_new_chunk: int,
                     n_new_chunks: int) -> torch.Tensor:
    """chunk_idx int32 [Hkv,n_sel] (contiguous, updated in place); base_chunk: the chunk that received the
    first token after the last rebuild."""
    if not chunk_idx.is_contiguous():
        raise ValueError("chunk_idx must be contiguous")
    _check(load_library().ts_chunk_list_admit(chunk_idx.data_ptr(), chunk_idx.shape[0], chunk_idx.shape[1],
                                              int(n_sink_chunks), int(base_chunk), int(first_new_chunk),
                                              int(n_new_chunks), _stream()),
           "ts_chunk_list_admit")
    return chunk_idx


def gather_chunks(k: torch.Tensor, v: torch.Tensor, chunk_idx: torch.Tensor, chunk_size: int):
    """-> (k_out, v_out) bf16 [Hkv, n_sel*chunk_size, 128]."""
    kv = _view(k, v)
    chunk_idx = chunk_idx.contiguous()
    n_sel = chunk_idx.shape[1]
    k_out = torch.empty(k.shape[0], n_sel * chunk_size, HEAD_DIM, dtype=k.dtype, device=k.device)
    v_out = torch.empty_like(k_out)
    _check(load_library().ts_gather_chunks(ctypes.byref(kv), chunk_idx.data_ptr(), n_sel, int(chunk_size),
                                           k_out.data_ptr(), v_out.data_ptr(), _stream()), "ts_gather_chunks")
    return k_out, v_out


def chunk_key_sums(k: torch.Tensor, chunk_size: int, out: Optional[torch.Tensor] = None,
                   chunk_begin: int = 0, chunk_end: Optional[int] = None) -> torch.Tensor:
    """k [Hkv,N,128] bf16 view -> ksum fp32 [Hkv, n_chunks(or more), 128]; only chunks
    [chunk_begin, chunk_end) are (re)computed."""
    kv = _view(k, None)
    n_chunks = (k.shape[1] + chunk_size - 1) // chunk_size if chunk_size > 0 else 0
    if out is None:
        out = torch.zeros(k.shape[0], max(n_chunks, 1), HEAD_DIM, dtype=torch.float32, device=k.device)
    if chunk_end is None:
        chunk_end = n_chunks
    _check(load_library().ts_chunk_key_sums(ctypes.byref(kv), int(chunk_size), int(chunk_begin), int(chunk_end),
                                            out.data_ptr(), out.stride(0), _stream()), "ts_chunk_key_sums")
    return out


def chunk_scores_from_sums(ksum: torch.Tensor, n_tokens: int, q: torch.Tensor, chunk_size: int, scale: float,
                           out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """ksum fp32 [Hkv, >=n_chunks, 128], q [Hq,128] bf16 -> scores fp32 [Hkv, ceil(n_tokens/chunk_size)]."""
    n_chunks = (n_tokens + chunk_size - 1) // chunk_size if chunk_size > 0 else 0
    q = q.contiguous()
    if out is None:
        out = torch.empty(ksum.shape[0], max(n_chunks, 1), dtype=torch.float32, device=ksum.device)
    _check(load_library().ts_chunk_scores_from_sums(ksum.data_ptr(), ksum.stride(0), ksum.shape[0], int(n_tokens),
                                                    q.data_ptr(), q.shape[0], int(chunk_size), float(scale),
                                                    out.data_ptr(), _stream()), "ts_chunk_scores_from_sums")
    return out


# ---- penalized probabilities and sampling ------------------------------------------------------------
SAMPLE_FULL, SAMPLE_MIN_P, SAMPLE_TOP_P, SAMPLE_ETA = 0, 1, 2, 3


def penalized_probs(logits: torch.Tensor, window: Optional[torch.Tensor], temperature: float, theta: float,
                    out: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """logits fp32 [R,V], window int32 [W] (device) or None -> probs fp32 [R,V] (Eq. 3)."""
    lib = load_library()
    if logits.dtype != torch.float32 or logits.dim() != 2 or not logits.is_contiguous():
        raise ValueError("logits must be a contiguous fp32 [rows, vocab] tensor")
    r, v = logits.shape
    nbytes = int(lib.ts_sampling_workspace_bytes(r, v))
    workspace = _workspace(nbytes, logits.device, workspace)
    if out is None:
        out = torch.empty_like(logits)
    n_window = 0 if window is None else int(window.numel())
    if window is not None:
        window = window.contiguous()
    _check(lib.ts_penalized_probs(logits.data_ptr(), r, v, window.data_ptr() if n_window else None, n_window,
                                  float(temperature), float(theta), out.data_ptr(), workspace.data_ptr(),
                                  workspace.numel(), _stream()), "ts_penalized_probs")
    return out


def sample_tokens(probs: torch.Tensor, method: int, param: float, u: torch.Tensor, want_pool: bool = False,
                  param2: float = 0.0):
    """probs fp32 [R,V], u fp32 [R] -> tokens int32 [R] (and (threshold, mass) fp32 [R] each)."""
    lib = load_library()
    if probs.dtype != torch.float32 or probs.dim() != 2 or not probs.is_contiguous():
        raise ValueError("probs must be a contiguous fp32 [rows, vocab] tensor")
    r, v = probs.shape
    u = u.contiguous()
    tokens = torch.empty(r, dtype=torch.int32, device=probs.device)
    thr = torch.empty(r, dtype=torch.float32, device=probs.device) if want_pool else None
    mass = torch.empty(r, dtype=torch.float32, device=probs.device) if want_pool else None
    _check(lib.ts_sample_tokens(probs.data_ptr(), r, v, int(method), float(param), float(param2), u.data_ptr(), tokens.data_ptr(),
                                thr.data_ptr() if want_pool else None, mass.data_ptr() if want_pool else None, _stream()),
           "ts_sample_tokens")
    return (tokens, thr, mass) if want_pool else tokens
