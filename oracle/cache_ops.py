"""CPU oracle for the cache maintenance around the attention passes -- TEST INFRASTRUCTURE ONLY.

Plain numpy, one obvious loop or indexing expression per definition; bf16 values are uint16 bit
patterns (copies move the bits untouched, sums widen them exactly to float64).  Shares nothing
with the GPU library.  Passages followed:
  append_accepted      Alg. 1, last step of the loop: C_full is updated with the accepted tokens.
  refresh_due          Alg. 1, the condition that guards the "Dynamic KV Cache Update" step: more than |B| - |S|
                       tokens were added since the last rebuild.
  chunk_list_admit     Sec. 3.3 "Dynamic KV Cache Updates": new tokens replace the least important
                       entries of C_p, from position |B|-1 towards |S| (here one chunk per entry, taken
                       when the chunk's first token arrives; a chunk is never listed twice).
  gather_chunks        Alg. 1: C_p = {C_full[0:|S|], Top-K(C_full)} as a buffer of its own.
  chunk_key_sums       (Eq. 2 is linear in the key) the per-chunk sums of the keys;
  scores_from_sums     Eq. 2 averaged per chunk, evaluated as (sum_j q_j) . (sum_t k_t) / |chunk|.
Pins: tests/test_cache_ops_pins.py.
"""
import numpy as np


def _widen(bits):
    b = np.ascontiguousarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def append_accepted(k, v, n_tokens, k_tree, v_tree, accepted):
    """k, v [Hkv, cap, d] u16 (modified copies are returned), k_tree/v_tree [T, Hkv, d] u16."""
    k, v = k.copy(), v.copy()
    for i, node in enumerate(accepted):
        for h in range(k.shape[0]):
            k[h, n_tokens + i] = k_tree[node, h]
            v[h, n_tokens + i] = v_tree[node, h]
    return k, v


def refresh_due(n_tokens, n_tokens_at_refresh, budget_tokens, sink_tokens):
    return (n_tokens - n_tokens_at_refresh) > (budget_tokens - sink_tokens)


def chunk_list_admit(chunk_idx, n_sink, base_chunk, first_new_chunk, n_new):
    """chunk_idx [Hkv, n_sel] int32: n_sink sink entries, then entries by decreasing importance; no chunk twice.

    New tokens enter C_p as they are generated and take its positions from the last one towards the
    sink.  At chunk granularity: base_chunk is the chunk that receives the first token generated after
    the last rebuild; chunk c (>= base_chunk) owns position n_sel - 1 - (c - base_chunk) from the moment
    its first token exists.  A chunk already listed (the partly filled last chunk, if the rebuild
    selected it) is not listed a second time: it trades places with the entry at its position, and
    nothing is evicted for it; a chunk among the sink entries stays where it is."""
    out = np.array(chunk_idx, dtype=np.int32, copy=True)
    n_sel = out.shape[1]
    assert n_new >= 0 and first_new_chunk >= base_chunk
    assert first_new_chunk + n_new - base_chunk <= n_sel - n_sink      # else a rebuild is due instead
    for h in range(out.shape[0]):
        for c in range(first_new_chunk, first_new_chunk + n_new):
            pos = n_sel - 1 - (c - base_chunk)
            where = [j for j in range(n_sel) if out[h, j] == c]
            assert len(where) <= 1
            if not where:
                out[h, pos] = c                    # evicts the least important entry still there
            elif where[0] >= n_sink and where[0] != pos:
                out[h, where[0]] = out[h, pos]
                out[h, pos] = c
    return out


def gather_chunks(k, v, chunk_idx, chunk):
    """k, v [Hkv, N, d] u16 -> (k_out, v_out) [Hkv, n_sel*chunk, d] u16, zero rows past the cache end."""
    hkv, n, d = k.shape
    n_sel = chunk_idx.shape[1]
    k_out = np.zeros((hkv, n_sel * chunk, d), dtype=np.uint16)
    v_out = np.zeros_like(k_out)
    for h in range(hkv):
        for j in range(n_sel):
            for w in range(chunk):
                t = int(chunk_idx[h, j]) * chunk + w
                if t < n:
                    k_out[h, j * chunk + w] = k[h, t]
                    v_out[h, j * chunk + w] = v[h, t]
    return k_out, v_out


def chunk_key_sums(k, chunk):
    """k [Hkv, N, d] u16 -> float64 [Hkv, ceil(N/chunk), d]."""
    hkv, n, d = k.shape
    n_chunks = (n + chunk - 1) // chunk
    kf = _widen(k)
    out = np.zeros((hkv, n_chunks, d), dtype=np.float64)
    for c in range(n_chunks):
        out[:, c, :] = kf[:, c * chunk:min(n, (c + 1) * chunk), :].sum(axis=1)
    return out


def scores_from_sums(ksum, n_tokens, q, chunk, scale):
    """ksum float [Hkv, n_chunks, d], q [Hq, d] u16 -> float64 [Hkv, n_chunks]."""
    hkv, n_chunks, d = ksum.shape
    qf = _widen(q)
    g = qf.shape[0] // hkv
    out = np.empty((hkv, n_chunks), dtype=np.float64)
    for h in range(hkv):
        qbar = qf[h * g:(h + 1) * g].sum(axis=0)
        for c in range(n_chunks):
            count = min(chunk, n_tokens - c * chunk)
            out[h, c] = scale * float(np.dot(qbar, np.asarray(ksum[h, c], dtype=np.float64))) / count
    return out
