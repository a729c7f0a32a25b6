"""Seeded synthetic inputs for the TokenSwift decode-attention hot path.

This module only makes inputs: KV caches, queries and draft trees with the shapes of the
models the paper evaluates (Sec. 4.1: YaRN-LLaMA2-7B-128k, LLaMA3.1-8B, Qwen2.5-1.5B/7B/14B).
They stand in for the caches that real generations on PG-19 prompts would produce; the
paper publishes no statistics of those, so values are N(0,1) rounded once to bf16, with a
number of "planted" chunks whose keys are shifted towards the query so that the top-k
selection has a recoverable answer.  Nothing here computes scores, softmax or attention.
Both the CPU oracle's tests and the GPU library's tests/benchmark take their inputs from
here, so both sides see the same bit patterns.

Two back ends with the same recipe: numpy (host, PCG64) for CPU tests and small parity cases,
torch (device generator) for caches too large to make on the host.  The discrete structure
(planted chunk ids, tree parents) always comes from numpy so it does not depend on the device.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, List, Optional

import numpy as np

HEAD_DIM = 128
CHUNK = 64


@dataclasses.dataclass(frozen=True)
class SynthConfig:
    name: str
    n_q_heads: int
    n_kv_heads: int
    n_tokens: int
    k: int                # selected chunks (beyond the sink)
    n_sink: int           # sink chunks always kept
    n_tree: int
    tree_kind: str        # "fixed" | "levels" | "random"
    n_layers: int
    seed: int
    n_planted: int        # planted chunks per KV head
    head_dim: int = HEAD_DIM
    chunk: int = CHUNK

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def n_chunks(self) -> int:
        return (self.n_tokens + self.chunk - 1) // self.chunk

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def n_sel(self) -> int:
        return self.n_sink + self.k


# The five workload shapes (index = position in the benchmark's config list).
CONFIGS: List[SynthConfig] = [
    SynthConfig("tiny", 4, 1, 4096, 8, 1, 8, "fixed", 1, 1001, 8),
    SynthConfig("qwen2.5-1.5b", 12, 2, 16384, 64, 1, 16, "levels", 28, 1002, 32),
    SynthConfig("llama3.1-8b", 32, 8, 65536, 64, 1, 32, "random", 32, 1003, 0),
    SynthConfig("yarn-llama2-7b-mha", 32, 32, 100000, 64, 1, 32, "random", 32, 1004, 16),
    SynthConfig("qwen2.5-14b", 40, 8, 102400, 128, 1, 64, "random", 48, 1005, 0),
]
CONFIG_BY_NAME: Dict[str, SynthConfig] = {c.name: c for c in CONFIGS}

TINY_PARENT = [-1, 0, 0, 1, 1, 2, 3, 4]


# ---------------------------------------------------------------------------------------------
# bf16 <-> fp32 bit conversions (round to nearest even), numpy
# ---------------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even), return the uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    rounded = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    out = np.where(nan, (u >> 16) | 0x0040, rounded).astype(np.uint16)
    return out


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


# ---------------------------------------------------------------------------------------------
# discrete structure
# ---------------------------------------------------------------------------------------------
def _rng(cfg: SynthConfig, layer: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([cfg.seed, layer, stream]))


def tree_parents(cfg: SynthConfig, layer: int = 0, n_tree: Optional[int] = None,
                 kind: Optional[str] = None) -> np.ndarray:
    """Parent array of the draft tree (App. E), topological order, -1 = root."""
    n_tree = cfg.n_tree if n_tree is None else n_tree
    kind = cfg.tree_kind if kind is None else kind
    rng = _rng(cfg, layer, 7)
    if kind == "fixed":
        if n_tree != len(TINY_PARENT):
            raise ValueError("the fixed tree has %d nodes" % len(TINY_PARENT))
        return np.asarray(TINY_PARENT, dtype=np.int32)
    if kind == "chain":
        return np.arange(-1, n_tree - 1, dtype=np.int32)
    if kind == "star":
        p = np.zeros(n_tree, dtype=np.int32)
        p[0] = -1
        return p
    if kind == "levels":
        # 4 draft positions with up to 4 candidates each: nodes of a level hang off random
        # nodes of the level before; the first level's nodes are roots.
        per = (n_tree + 3) // 4
        p = np.empty(n_tree, dtype=np.int32)
        for i in range(n_tree):
            lvl = i // per
            if lvl == 0:
                p[i] = -1
            else:
                lo, hi = (lvl - 1) * per, min(lvl * per, n_tree)
                p[i] = rng.integers(lo, hi)
        return p
    if kind == "random":
        p = np.empty(n_tree, dtype=np.int32)
        p[0] = -1
        for i in range(1, n_tree):
            p[i] = rng.integers(0, i)
        return p
    raise ValueError("unknown tree kind %r" % kind)


def planted_chunks(cfg: SynthConfig, layer: int = 0, n_tokens: Optional[int] = None,
                   n_planted: Optional[int] = None) -> np.ndarray:
    """[n_kv_heads, n_planted] distinct chunk ids (never a sink chunk) to shift towards q."""
    n_tokens = cfg.n_tokens if n_tokens is None else n_tokens
    n_planted = cfg.n_planted if n_planted is None else n_planted
    n_chunks = (n_tokens + cfg.chunk - 1) // cfg.chunk
    rng = _rng(cfg, layer, 11)
    n_planted = min(n_planted, max(n_chunks - cfg.n_sink, 0))
    out = np.empty((cfg.n_kv_heads, n_planted), dtype=np.int64)
    for h in range(cfg.n_kv_heads):
        out[h] = np.sort(rng.choice(np.arange(cfg.n_sink, n_chunks), size=n_planted, replace=False))
    return out


# ---------------------------------------------------------------------------------------------
# numpy back end
# ---------------------------------------------------------------------------------------------
def make_layer(cfg: SynthConfig, layer: int = 0, n_tokens: Optional[int] = None,
               n_tree: Optional[int] = None, tree_kind: Optional[str] = None) -> dict:
    """One layer's inputs as numpy uint16 (bf16 bits) arrays.

    q [Hq,d]; q_tree [T,Hq,d] with q_tree[0] = q; k_tree, v_tree [T,Hkv,d]; k, v [Hkv,N,d];
    parent [T] int32; planted [Hkv, n_planted] chunk ids.
    """
    n_tokens = cfg.n_tokens if n_tokens is None else n_tokens
    n_tree = cfg.n_tree if n_tree is None else n_tree
    d, hq, hkv, g = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads, cfg.group
    rng = _rng(cfg, layer, 1)
    q = f32_to_bf16_bits(rng.standard_normal((hq, d), dtype=np.float32))
    q_tree = f32_to_bf16_bits(rng.standard_normal((n_tree, hq, d), dtype=np.float32))
    q_tree[0] = q      # tree node 0 is the token the iteration starts from: the query of the draft pass and of the scores
    k_tree = f32_to_bf16_bits(rng.standard_normal((n_tree, hkv, d), dtype=np.float32))
    v_tree = f32_to_bf16_bits(rng.standard_normal((n_tree, hkv, d), dtype=np.float32))
    k = rng.standard_normal((hkv, n_tokens, d), dtype=np.float32)
    v = f32_to_bf16_bits(rng.standard_normal((hkv, n_tokens, d), dtype=np.float32))
    planted = planted_chunks(cfg, layer, n_tokens)
    if planted.shape[1] > 0:
        qdir = bf16_bits_to_f32(q).reshape(hkv, g, d).sum(axis=1)
        qdir /= np.linalg.norm(qdir, axis=1, keepdims=True)
        for h in range(hkv):
            for c in planted[h]:
                lo, hi = c * cfg.chunk, min((c + 1) * cfg.chunk, n_tokens)
                k[h, lo:hi] += np.float32(0.5) * qdir[h]
    k = f32_to_bf16_bits(k)
    parent = tree_parents(cfg, layer, n_tree, tree_kind)
    return dict(q=q, q_tree=q_tree, k_tree=k_tree, v_tree=v_tree, k=k, v=v, parent=parent,
                planted=planted)


# ---------------------------------------------------------------------------------------------
# torch back end (bulk data made on the device; same recipe)
# ---------------------------------------------------------------------------------------------
def make_layer_torch(cfg: SynthConfig, layer: int, device, n_tokens: Optional[int] = None,
                     n_tree: Optional[int] = None, tree_kind: Optional[str] = None) -> dict:
    """Same as make_layer, as torch bfloat16 tensors on `device` (parent, planted stay numpy)."""
    import torch

    n_tokens = cfg.n_tokens if n_tokens is None else n_tokens
    n_tree = cfg.n_tree if n_tree is None else n_tree
    d, hq, hkv, g = cfg.head_dim, cfg.n_q_heads, cfg.n_kv_heads, cfg.group
    gen = torch.Generator(device=device)
    gen.manual_seed(cfg.seed * 1000003 + layer)

    def normal(*shape):
        return torch.randn(*shape, generator=gen, device=device, dtype=torch.float32)

    q = normal(hq, d).to(torch.bfloat16)
    q_tree = normal(n_tree, hq, d).to(torch.bfloat16)
    q_tree[0] = q      # tree node 0 is the token the iteration starts from: the query of the draft pass and of the scores
    k_tree = normal(n_tree, hkv, d).to(torch.bfloat16)
    v_tree = normal(n_tree, hkv, d).to(torch.bfloat16)
    k = torch.empty(hkv, n_tokens, d, device=device, dtype=torch.bfloat16)
    v = torch.empty(hkv, n_tokens, d, device=device, dtype=torch.bfloat16)
    planted = planted_chunks(cfg, layer, n_tokens)
    qdir = q.float().reshape(hkv, g, d).sum(dim=1)
    qdir = qdir / qdir.norm(dim=1, keepdim=True)
    for h in range(hkv):  # head by head keeps the fp32 staging buffer small
        kh = normal(n_tokens, d)
        for c in planted[h]:
            lo, hi = int(c) * cfg.chunk, min((int(c) + 1) * cfg.chunk, n_tokens)
            kh[lo:hi] += 0.5 * qdir[h]
        k[h] = kh.to(torch.bfloat16)
        v[h] = normal(n_tokens, d).to(torch.bfloat16)
    parent = tree_parents(cfg, layer, n_tree, tree_kind)
    return dict(q=q, q_tree=q_tree, k_tree=k_tree, v_tree=v_tree, k=k, v=v, parent=parent,
                planted=planted)


def torch_bf16_to_bits(t) -> np.ndarray:
    """torch bfloat16 tensor (any device) -> numpy uint16 bit patterns on the host."""
    import torch

    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_torch_bf16(b: np.ndarray, device):
    """numpy uint16 bit patterns -> torch bfloat16 tensor on `device`."""
    import torch

    t = torch.from_numpy(np.ascontiguousarray(b).view(np.int16).copy())
    return t.to(device).view(torch.bfloat16)
