"""Plain numpy/scipy building blocks used by the tests to state what the paper and the
mathematics fix, independently of both the oracle's C code and the GPU library."""
import numpy as np
from scipy.special import logsumexp, softmax

import ts_synth as S


def widen(bits):
    return S.bf16_bits_to_f64(bits)


def rand_bits(rng, *shape, scale=1.0):
    return S.f32_to_bf16_bits((rng.standard_normal(shape) * scale).astype(np.float32))


def dense_attention(q, keys, vals, scale, mask=None):
    """Textbook softmax attention with library routines. q [R,d], keys/vals [M,d] float64,
    mask [R,M] bool (True = may attend). Returns (out [R,d], lse [R])."""
    z = scale * (q @ keys.T)
    if mask is not None:
        z = np.where(mask, z, -np.inf)
    p = softmax(z, axis=-1)
    return p @ vals, logsumexp(z, axis=-1)


def ancestors_or_self(parent, i):
    out = []
    u = int(i)
    while u != -1:
        out.append(u)
        u = int(parent[u])
    return out


def err_metrics(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    max_abs = float(np.max(np.abs(got - ref))) if got.size else 0.0
    denom = float(np.linalg.norm(ref.ravel()))
    rel_l2 = float(np.linalg.norm((got - ref).ravel()) / denom) if denom > 0 else max_abs
    return max_abs, rel_l2
