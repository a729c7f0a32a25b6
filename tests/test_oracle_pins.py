"""Pins of the fp64 oracle against what the paper and the mathematics fix (CPU only).

The paper prints no worked numeric example of scoring, selection or attention (all of its
numbers are end-to-end acceptance rates and latencies), so the pins are closed forms,
special cases that reduce to library routines (scipy softmax / numpy matmul / Python's
sort), invariants and brute force on tiny inputs.  Each is chosen so that a plausible
mistake in the oracle (dropped scale, wrong group mapping, off-by-one in a chunk range,
mask transposed, self not included, ...) fails at least one of them.
"""
import math
import os

import numpy as np
import pytest

import oracle
import ts_synth as S
from helpers import ancestors_or_self, dense_attention, rand_bits, widen

D = 128
SCALE = 1.0 / math.sqrt(D)
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _cache(rng, hkv, n, d=D, vscale=1.0):
    return rand_bits(rng, hkv, n, d), rand_bits(rng, hkv, n, d, scale=vscale)


# ------------------------------------------------------------------------------------------
# chunk scores (Eq. 2)
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("hq,hkv,n,chunk", [(4, 1, 200, 64), (12, 2, 257, 64), (5, 1, 64, 16),
                                            (32, 32, 130, 64), (6, 3, 63, 64)])
def test_scores_equal_summed_query_dot_mean_key(hq, hkv, n, chunk):
    """Eq. 2 is linear: sum_j q_j.k == (sum_j q_j).k, and the chunk mean of dots is the dot
    with the chunk-mean key.  Computed here with numpy reductions only."""
    rng = np.random.default_rng(1)
    q = rand_bits(rng, hq, D)
    k, _ = _cache(rng, hkv, n)
    got = oracle.chunk_scores(q, k, chunk, SCALE)
    g = hq // hkv
    qbar = widen(q).reshape(hkv, g, D).sum(axis=1)
    n_chunks = -(-n // chunk)
    assert got.shape == (hkv, n_chunks)
    for h in range(hkv):
        for c in range(n_chunks):
            kmean = widen(k[h, c * chunk:min(n, (c + 1) * chunk)]).mean(axis=0)
            assert got[h, c] == pytest.approx(SCALE * float(qbar[h] @ kmean), rel=1e-12, abs=1e-12)


def test_scores_equal_replicated_key_formulation():
    """The paper contrasts Eq. 2 with replicating K for each query head of the group
    (Sec. 3.3); summing the replicated per-head scores must give the same number."""
    rng = np.random.default_rng(2)
    hq, hkv, n = 12, 3, 96
    q = rand_bits(rng, hq, D)
    k, _ = _cache(rng, hkv, n)
    got = oracle.chunk_scores(q, k, 1, 1.0)            # chunk = 1: per-token, raw Q.K^T
    g = hq // hkv
    k_rep = np.repeat(widen(k), g, axis=0)             # [hq, n, d]
    per_head = np.einsum("jd,jnd->jn", widen(q), k_rep)
    want = per_head.reshape(hkv, g, n).sum(axis=1)
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_scores_mha_is_plain_qk():
    """g = 1: the score is the plain dot product Q K^T (Sec. 3.3, first sentence)."""
    rng = np.random.default_rng(3)
    q = rand_bits(rng, 4, D)
    k, _ = _cache(rng, 4, 50)
    got = oracle.chunk_scores(q, k, 1, 1.0)
    want = np.einsum("hd,hnd->hn", widen(q), widen(k))
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_scores_hand_values():
    """Integers small enough to check by hand: q_0 = e_0 + 2 e_1, q_1 = 3 e_0, one KV head,
    keys k_t = (t+1) e_0 + e_1.  Per-token score = (1+3)(t+1) + 2 = 4t + 6.
    chunk 2 over 5 tokens -> means (6+10)/2, (14+18)/2, 22; times scale 0.5."""
    q = np.zeros((2, D), dtype=np.float32)
    q[0, 0], q[0, 1], q[1, 0] = 1, 2, 3
    k = np.zeros((1, 5, D), dtype=np.float32)
    for t in range(5):
        k[0, t, 0], k[0, t, 1] = t + 1, 1
    got = oracle.chunk_scores(S.f32_to_bf16_bits(q), S.f32_to_bf16_bits(k), 2, 0.5)
    np.testing.assert_array_equal(got, np.array([[4.0, 8.0, 11.0]]))


def test_scores_respect_strides():
    """A token-major cache [N, Hkv, d] viewed as [Hkv, N, d] gives the same scores."""
    rng = np.random.default_rng(4)
    q = rand_bits(rng, 4, D)
    k_tm = rand_bits(rng, 70, 2, D)                   # token-major storage
    view = k_tm.transpose(1, 0, 2)                    # strided [Hkv, N, d] view
    got = oracle.chunk_scores(q, view, 64, SCALE)
    want = oracle.chunk_scores(q, np.ascontiguousarray(view), 64, SCALE)
    np.testing.assert_array_equal(got, want)


# ------------------------------------------------------------------------------------------
# top-k chunks
# ------------------------------------------------------------------------------------------
def _brute_topk(scores_row, n_sink, k):
    """Python's sort with the explicit key (score descending, index ascending, NaN last)."""
    cand = list(range(n_sink, len(scores_row)))
    def key(c):
        s = float(scores_row[c])
        return (1, 0.0, c) if math.isnan(s) else (0, -s if s != 0 else 0.0, c)
    cand.sort(key=key)
    return list(range(n_sink)) + cand[:k]


@pytest.mark.parametrize("seed", range(6))
def test_topk_matches_sort(seed):
    rng = np.random.default_rng(100 + seed)
    hkv, n_chunks = 3, int(rng.integers(2, 33))
    n_sink = int(rng.integers(0, min(3, n_chunks)))
    k = int(rng.integers(0 if n_sink else 1, n_chunks - n_sink + 1))
    scores = rng.standard_normal((hkv, n_chunks)).astype(np.float32)
    scores[:, ::3] = np.round(scores[:, ::3])          # planted ties
    got = oracle.topk_chunks(scores, n_sink, k)
    for h in range(hkv):
        assert got[h].tolist() == _brute_topk(scores[h], n_sink, k)


def test_topk_ties_zeros_nan():
    s = np.array([[5.0, 1.0, 1.0, -0.0, 0.0, np.nan, 1.0, np.nan, -np.inf, np.inf]], dtype=np.float32)
    got = oracle.topk_chunks(s, 1, 9)[0].tolist()
    # sink 0; then inf(9); the three 1.0 by index (1,2,6); the zeros by index (3,4) since
    # -0 == +0; -inf (8); NaNs last by index (5,7)
    assert got == [0, 9, 1, 2, 6, 3, 4, 8, 5, 7]
    assert got == _brute_topk(s[0], 1, 9)


def test_topk_all_equal_and_structure():
    """All scores equal: selection is the lowest indices in order.  The sink chunks always
    lead, selected ones are distinct, none is a sink chunk, |C_p| = n_sink + k."""
    s = np.full((2, 17), 0.25, dtype=np.float32)
    got = oracle.topk_chunks(s, 2, 6)
    assert got.tolist() == [[0, 1, 2, 3, 4, 5, 6, 7]] * 2
    rng = np.random.default_rng(7)
    s = rng.standard_normal((4, 40)).astype(np.float32)
    got = oracle.topk_chunks(s, 3, 10)
    for h in range(4):
        row = got[h].tolist()
        assert row[:3] == [0, 1, 2] and len(set(row)) == 13 and min(row[3:]) >= 3
        sel = s[h][row[3:]]
        assert np.all(np.diff(sel) <= 0)                              # decreasing importance
        rest = np.delete(s[h], row)
        assert rest.size == 0 or rest.max() <= sel.min()              # nothing better left out


def test_topk_rejects_bad_arguments():
    s = np.zeros((1, 4), dtype=np.float32)
    with pytest.raises(ValueError):
        oracle.topk_chunks(s, 2, 3)      # 2 + 3 > 4 chunks
    with pytest.raises(ValueError):
        oracle.topk_chunks(s, 0, 0)      # empty selection


# ------------------------------------------------------------------------------------------
# partial-KV attention
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("hq,hkv,n,chunk", [(4, 1, 256, 64), (12, 2, 200, 64), (5, 1, 33, 16),
                                            (8, 8, 65, 64), (6, 3, 1, 64)])
def test_partial_with_all_chunks_is_full_attention(hq, hkv, n, chunk):
    """Listing every chunk must give ordinary attention over tokens 0..N-1 (scipy softmax),
    including a short last chunk."""
    rng = np.random.default_rng(11)
    q = rand_bits(rng, hq, D)
    k, v = _cache(rng, hkv, n)
    n_chunks = -(-n // chunk)
    idx = np.tile(np.arange(n_chunks, dtype=np.int32), (hkv, 1))
    out, lse = oracle.partial_attn(q, k, v, idx, chunk, SCALE)
    g = hq // hkv
    for j in range(hq):
        want, wlse = dense_attention(widen(q[j:j + 1]), widen(k[j // g]), widen(v[j // g]), SCALE)
        np.testing.assert_allclose(out[j], want[0], rtol=1e-11, atol=1e-12)
        assert lse[j] == pytest.approx(wlse[0], rel=1e-12)


def test_partial_subset_and_order_invariance():
    """A strict subset of chunks equals dense attention over exactly those token ranges, and
    the order in which chunks are listed does not matter."""
    rng = np.random.default_rng(12)
    hq, hkv, n, chunk = 8, 2, 300, 64                   # 5 chunks, last has 44 tokens
    q = rand_bits(rng, hq, D)
    k, v = _cache(rng, hkv, n)
    idx = np.array([[0, 4, 2], [3, 0, 4]], dtype=np.int32)
    out, lse = oracle.partial_attn(q, k, v, idx, chunk, SCALE)
    for j in range(hq):
        h = j // 4
        toks = np.concatenate([np.arange(c * chunk, min(n, (c + 1) * chunk)) for c in idx[h]])
        want, wlse = dense_attention(widen(q[j:j + 1]), widen(k[h][toks]), widen(v[h][toks]), SCALE)
        np.testing.assert_allclose(out[j], want[0], rtol=1e-11, atol=1e-12)
        assert lse[j] == pytest.approx(wlse[0], rel=1e-12)
    out2, _ = oracle.partial_attn(q, k, v, idx[:, ::-1].copy(), chunk, SCALE)
    np.testing.assert_allclose(out2, out, rtol=0, atol=1e-12)


def test_partial_zero_query_is_mean_of_selected_values():
    """q = 0 makes every probability 1/|keys|: the output is the arithmetic mean of V over the
    selected tokens -- pins which tokens a chunk id names (44-token last chunk included)."""
    rng = np.random.default_rng(13)
    hkv, n, chunk = 2, 300, 64
    q = np.zeros((4, D), dtype=np.uint16)
    k, v = _cache(rng, hkv, n)
    idx = np.array([[1, 4], [4, 0]], dtype=np.int32)
    out, lse = oracle.partial_attn(q, k, v, idx, chunk, SCALE)
    for j in range(4):
        h = j // 2
        toks = np.concatenate([np.arange(c * chunk, min(n, (c + 1) * chunk)) for c in idx[h]])
        np.testing.assert_allclose(out[j], widen(v[h][toks]).mean(axis=0), rtol=1e-12, atol=1e-13)
        assert lse[j] == pytest.approx(math.log(len(toks)), rel=1e-13)


def test_single_key_returns_value_exactly():
    rng = np.random.default_rng(14)
    q = rand_bits(rng, 4, D)
    k, v = _cache(rng, 2, 1)
    out, _ = oracle.partial_attn(q, k, v, np.zeros((2, 1), dtype=np.int32), 64, SCALE)
    for j in range(4):
        np.testing.assert_array_equal(out[j], widen(v[j // 2, 0]))


def test_two_key_closed_form():
    """Two keys with logits 0 and x: p = (1/(1+e^x), e^x/(1+e^x)).  Values from the text
    fixture, which lists x and the probabilities from the logistic closed form."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "two_key_softmax.txt"))
            if l.strip() and not l.startswith("#")]
    for a, b, scale, p1_want in [(float(r[0]), float(r[1]), float(r[2]), float(r[3])) for r in rows]:
        q = np.zeros((1, D), dtype=np.float32); q[0, 5] = a
        k = np.zeros((1, 2, D), dtype=np.float32); k[0, 1, 5] = b; k[0, 1, 6] = 7.0  # 6 is ignored by q
        v = np.zeros((1, 2, D), dtype=np.float32); v[0, 0, 0] = 1.0; v[0, 1, 1] = 1.0
        out, lse = oracle.partial_attn(S.f32_to_bf16_bits(q), S.f32_to_bf16_bits(k),
                                       S.f32_to_bf16_bits(v), np.zeros((1, 1), np.int32), 64, scale)
        assert out[0, 1] == pytest.approx(p1_want, rel=1e-9)
        assert out[0, 0] == pytest.approx(1.0 - p1_want, rel=1e-9, abs=1e-15)
        assert lse[0] == pytest.approx(math.log1p(math.exp(scale * a * b)), rel=1e-12)


def test_softmax_rows_sum_to_one_via_lse():
    """exp(logit - lse) summed over the key set is 1; logits recomputed with numpy."""
    rng = np.random.default_rng(15)
    hq, hkv, n = 4, 2, 150
    q = rand_bits(rng, hq, D)
    k, v = _cache(rng, hkv, n)
    idx = np.tile(np.arange(3, dtype=np.int32), (hkv, 1))
    out, lse = oracle.partial_attn(q, k, v, idx, 64, SCALE)
    for j in range(hq):
        z = SCALE * widen(k[j // 2]) @ widen(q[j])
        p = np.exp(z - lse[j])
        assert abs(p.sum() - 1.0) < 1e-13 and np.all(p >= 0)
        np.testing.assert_allclose(out[j], p @ widen(v[j // 2]), rtol=1e-11, atol=1e-13)


def test_logit_shift_invariance_and_large_logits():
    """Adding c*q/|q|^2-like shifts that move every logit by the same constant leaves the
    output unchanged; logits near +-60 do not overflow (max subtraction)."""
    rng = np.random.default_rng(16)
    n = 40
    q = np.zeros((1, D), dtype=np.float32); q[0, 0] = 8.0
    kf = (rng.standard_normal((1, n, D)) * 4).astype(np.float32)
    kf[0, :, 0] = np.round(kf[0, :, 0])                  # integers: the shifted values stay exact in bf16
    v = rand_bits(rng, 1, n, D)
    idx = np.zeros((1, 1), dtype=np.int32)
    out0, lse0 = oracle.partial_attn(S.f32_to_bf16_bits(q), S.f32_to_bf16_bits(kf), v, idx, 64, 1.0)
    kf2 = kf.copy(); kf2[0, :, 0] += 64.0                 # every logit + 512
    kb, kb2 = S.f32_to_bf16_bits(kf), S.f32_to_bf16_bits(kf2)
    # the shift must be exact in bf16 for the identity to be exact
    assert np.array_equal(widen(kb2)[0, :, 0] - widen(kb)[0, :, 0], np.full(n, 64.0))
    out1, lse1 = oracle.partial_attn(S.f32_to_bf16_bits(q), kb2, v, idx, 64, 1.0)
    np.testing.assert_allclose(out1, out0, rtol=1e-12, atol=1e-13)
    assert lse1[0] == pytest.approx(lse0[0] + 512.0, rel=1e-13)
    assert np.all(np.isfinite(out1))


# ------------------------------------------------------------------------------------------
# tree verification attention (App. E)
# ------------------------------------------------------------------------------------------
def _tree_inputs(rng, t, hq, hkv, n):
    q_tree = rand_bits(rng, t, hq, D)
    k_tree = rand_bits(rng, t, hkv, D)
    v_tree = rand_bits(rng, t, hkv, D)
    k, v = _cache(rng, hkv, n)
    return q_tree, k_tree, v_tree, k, v


@pytest.mark.parametrize("hq,hkv,n,t", [(4, 1, 100, 8), (12, 2, 65, 5), (4, 4, 0, 6), (5, 1, 1, 1)])
def test_chain_tree_is_causal_attention(hq, hkv, n, t):
    """A linear chain is ordinary causal decoding of t tokens after an n-token cache: row i sees
    the cache and tree tokens 0..i (lower-triangular mask, numpy tril + scipy softmax)."""
    rng = np.random.default_rng(21)
    q_tree, k_tree, v_tree, k, v = _tree_inputs(rng, t, hq, hkv, n)
    parent = np.arange(-1, t - 1, dtype=np.int32)
    out, lse = oracle.tree_verify(q_tree, k if n else None, v if n else None, k_tree, v_tree, parent, SCALE)
    g = hq // hkv
    mask = np.concatenate([np.ones((t, n), bool), np.tril(np.ones((t, t), bool))], axis=1)
    for j in range(hq):
        h = j // g
        keys = np.concatenate([widen(k[h]), widen(k_tree[:, h])], axis=0)
        vals = np.concatenate([widen(v[h]), widen(v_tree[:, h])], axis=0)
        want, wlse = dense_attention(widen(q_tree[:, j]), keys, vals, SCALE, mask)
        np.testing.assert_allclose(out[:, j], want, rtol=1e-11, atol=1e-12)
        np.testing.assert_allclose(lse[:, j], wlse, rtol=1e-12)


@pytest.mark.parametrize("kind,t", [("fixed", 8), ("random", 13), ("levels", 16), ("star", 7)])
def test_every_root_path_is_causal_attention(kind, t):
    """Lossless verification (Sec. 3.1): the row of node i must be what plain causal decoding of
    the token sequence root..i would give.  Each path is extracted and run through dense
    attention over [cache, path]."""
    rng = np.random.default_rng(22)
    hq, hkv, n = 6, 2, 70
    q_tree, k_tree, v_tree, k, v = _tree_inputs(rng, t, hq, hkv, n)
    parent = S.tree_parents(S.CONFIGS[0], 0, t, kind)
    out, lse = oracle.tree_verify(q_tree, k, v, k_tree, v_tree, parent, SCALE)
    for i in range(t):
        path = ancestors_or_self(parent, i)[::-1]        # root .. i
        for j in range(hq):
            h = j // 3
            keys = np.concatenate([widen(k[h]), widen(k_tree[path, h])], axis=0)
            vals = np.concatenate([widen(v[h]), widen(v_tree[path, h])], axis=0)
            want, wlse = dense_attention(widen(q_tree[i, j])[None], keys, vals, SCALE)
            np.testing.assert_allclose(out[i, j], want[0], rtol=1e-11, atol=1e-12)
            assert lse[i, j] == pytest.approx(wlse[0], rel=1e-12)


def test_sibling_isolation_is_bit_exact():
    """Changing K/V of a node that is not an ancestor of i (a sibling, a descendant, a cousin)
    must not change row i at all; changing an ancestor or i itself must."""
    rng = np.random.default_rng(23)
    t, hq, hkv, n = 8, 4, 1, 50
    q_tree, k_tree, v_tree, k, v = _tree_inputs(rng, t, hq, hkv, n)
    parent = np.asarray(S.TINY_PARENT, dtype=np.int32)
    base, _ = oracle.tree_verify(q_tree, k, v, k_tree, v_tree, parent, SCALE)
    for u in range(t):
        k2, v2 = k_tree.copy(), v_tree.copy()
        k2[u] = rand_bits(rng, hkv, D)
        v2[u] = rand_bits(rng, hkv, D)
        pert, _ = oracle.tree_verify(q_tree, k, v, k2, v2, parent, SCALE)
        for i in range(t):
            visible = u in ancestors_or_self(parent, i)
            same = np.array_equal(pert[i], base[i])
            assert same != visible, (u, i)


def test_tree_zero_query_is_mean_over_cache_and_ancestors():
    rng = np.random.default_rng(24)
    t, hq, hkv, n = 8, 2, 2, 37
    _, k_tree, v_tree, k, v = _tree_inputs(rng, t, hq, hkv, n)
    q_tree = np.zeros((t, hq, D), dtype=np.uint16)
    parent = np.asarray(S.TINY_PARENT, dtype=np.int32)
    out, lse = oracle.tree_verify(q_tree, k, v, k_tree, v_tree, parent, SCALE)
    for i in range(t):
        anc = ancestors_or_self(parent, i)
        for j in range(hq):
            vals = np.concatenate([widen(v[j]), widen(v_tree[anc, j])], axis=0)
            np.testing.assert_allclose(out[i, j], vals.mean(axis=0), rtol=1e-12, atol=1e-13)
            assert lse[i, j] == pytest.approx(math.log(n + len(anc)), rel=1e-13)


def test_tree_single_node_no_cache_returns_value():
    rng = np.random.default_rng(25)
    q_tree, k_tree, v_tree, _, _ = _tree_inputs(rng, 1, 4, 2, 1)
    out, _ = oracle.tree_verify(q_tree, None, None, k_tree, v_tree, np.array([-1], np.int32), SCALE)
    for j in range(4):
        np.testing.assert_array_equal(out[0, j], widen(v_tree[0, j // 2]))


def test_tree_row_selection_matches_full():
    rng = np.random.default_rng(26)
    t, hq, hkv, n = 8, 4, 2, 90
    q_tree, k_tree, v_tree, k, v = _tree_inputs(rng, t, hq, hkv, n)
    parent = np.asarray(S.TINY_PARENT, dtype=np.int32)
    full, flse = oracle.tree_verify(q_tree, k, v, k_tree, v_tree, parent, SCALE)
    rows = [(7, 3), (0, 0), (4, 2)]
    sub, slse = oracle.tree_verify(q_tree, k, v, k_tree, v_tree, parent, SCALE, rows=rows)
    for r, (i, j) in enumerate(rows):
        np.testing.assert_array_equal(sub[r], full[i, j])
        assert slse[r] == flse[i, j]


def test_tree_rejects_bad_parent():
    rng = np.random.default_rng(27)
    q_tree, k_tree, v_tree, k, v = _tree_inputs(rng, 3, 2, 1, 4)
    for bad in ([0, 0, 1], [-1, 1, 0], [-1, 0, 2], [-2, 0, 0]):
        with pytest.raises(ValueError):
            oracle.tree_verify(q_tree, k, v, k_tree, v_tree, np.array(bad, np.int32), SCALE)


# ------------------------------------------------------------------------------------------
# combine identity (split-K) and end-to-end sanity of the generator
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("cuts", [(0, 17, 40), (0, 1, 2, 40), (0, 40), (0, 13, 13, 40)])
def test_combine_of_partials_is_attention_over_union(cuts):
    rng = np.random.default_rng(31)
    n = cuts[-1]
    q = rand_bits(rng, 1, D)
    k, v = _cache(rng, 1, n, vscale=3.0)
    z = SCALE * widen(k[0]) @ widen(q[0])
    ms, ls, os_ = [], [], []
    for a, b in zip(cuts[:-1], cuts[1:]):
        if a == b:
            ms.append(-np.inf); ls.append(0.0); os_.append(np.zeros(D))
            continue
        m = z[a:b].max()
        w = np.exp(z[a:b] - m)
        ms.append(m); ls.append(w.sum()); os_.append(w @ widen(v[0, a:b]))
    got, glse = oracle.combine(ms, ls, np.stack(os_))
    want, wlse = oracle.partial_attn(q, k, v, np.zeros((1, 1), np.int32), 64, SCALE)
    np.testing.assert_allclose(got, want[0], rtol=1e-12, atol=1e-13)
    assert glse == pytest.approx(wlse[0], rel=1e-13)


@pytest.mark.parametrize("ci", [0, 1])
def test_planted_chunks_stand_out(ci):
    """Generator + Eq. 2 + top-k end to end: planted chunks score higher by about
    0.5*scale*|sum_j q_j|, and most of them are selected."""
    cfg = S.CONFIGS[ci]
    x = S.make_layer(cfg, 0)
    sc = oracle.chunk_scores(x["q"], x["k"], cfg.chunk, cfg.scale)
    idx = oracle.topk_chunks(sc, cfg.n_sink, cfg.k)
    qbar = widen(x["q"]).reshape(cfg.n_kv_heads, cfg.group, -1).sum(axis=1)
    for h in range(cfg.n_kv_heads):
        planted = set(x["planted"][h].tolist())
        others = [c for c in range(cfg.n_sink, cfg.n_chunks) if c not in planted]
        shift = sc[h][sorted(planted)].mean() - sc[h][others].mean()
        want = 0.5 * cfg.scale * np.linalg.norm(qbar[h])
        sigma = cfg.scale * np.linalg.norm(qbar[h]) / math.sqrt(cfg.chunk)
        assert abs(shift - want) < 4 * sigma / math.sqrt(len(planted))
        hit = len(planted & set(idx[h, cfg.n_sink:].tolist()))
        assert hit >= 0.6 * min(len(planted), cfg.k)
        assert idx[h, 0] == 0
