"""Pins of the cache-maintenance oracle (CPU only): each definition against what the paper and the
mathematics fix, by means other than the oracle's own expression."""
import numpy as np
import pytest

import oracle
from oracle import cache_ops as C
from helpers import rand_bits, widen

D = 128


def test_append_accepted_places_the_accepted_path_after_the_cache():
    rng = np.random.default_rng(1)
    hkv, cap, n, t = 3, 40, 17, 9
    k, v = rand_bits(rng, hkv, cap, D), rand_bits(rng, hkv, cap, D)
    kt, vt = rand_bits(rng, t, hkv, D), rand_bits(rng, t, hkv, D)
    acc = [0, 2, 5, 8]
    k2, v2 = C.append_accepted(k, v, n, kt, vt, acc)
    # untouched: everything before n and after n + len(acc)
    assert np.array_equal(k2[:, :n], k[:, :n]) and np.array_equal(v2[:, n + 4:], v[:, n + 4:])
    # the appended block is the tree rows in path order, head-major (an indexing identity)
    assert np.array_equal(k2[:, n:n + 4], kt[acc].transpose(1, 0, 2))
    assert np.array_equal(v2[:, n:n + 4], vt[acc].transpose(1, 0, 2))
    # attending over the grown cache == tree verification of the accepted chain: the property
    # that makes the accepted tokens ordinary cache entries for the next step (Alg. 1)
    q = rand_bits(rng, 1, hkv, D)
    out_a, _ = oracle.partial_attn(q[0], k2[:, :n + 4], v2[:, :n + 4], np.zeros((hkv, 1), np.int32), 64, 0.1)
    chain = np.arange(-1, 3, dtype=np.int32)
    qt = np.concatenate([rand_bits(rng, 3, hkv, D), q], axis=0)          # last node carries q
    out_b, _ = oracle.tree_verify(qt, k[:, :n], v[:, :n], kt[acc], vt[acc], chain, 0.1)
    np.testing.assert_allclose(out_a, out_b[3], rtol=0, atol=1e-12)


def test_refresh_due_matches_the_loop_condition_of_alg1():
    # |B| = 4096, |S| = 64: a rebuild is due once more than |B| - |S| tokens were added since e
    assert not C.refresh_due(10000 + 4032, 10000, 4096, 64)
    assert C.refresh_due(10000 + 4033, 10000, 4096, 64)
    assert not C.refresh_due(5, 5, 4096, 64)
    # walking the loop: the number of rebuilds over a run equals floor-style counting by hand
    e, rebuilds = 100, 0
    for n in range(100, 1000):
        if C.refresh_due(n, e, 200, 10):
            e, rebuilds = n, rebuilds + 1
    assert rebuilds == (999 - 100) // 191          # every 191 = (|B|-|S|) + 1 tokens


def test_chunk_list_admit_evicts_from_the_tail_towards_the_sink():
    idx = np.array([[0, 7, 3, 9, 5], [0, 2, 8, 4, 6]], dtype=np.int32)   # sink 0, then decreasing importance
    out = C.chunk_list_admit(idx, 1, 20, 20, 2)
    assert out.tolist() == [[0, 7, 3, 21, 20], [0, 2, 8, 21, 20]]
    assert np.array_equal(C.chunk_list_admit(idx, 1, 20, 20, 0), idx)
    full = C.chunk_list_admit(idx, 1, 30, 30, 4)
    assert full[:, 0].tolist() == [0, 0] and sorted(full[0, 1:].tolist()) == [30, 31, 32, 33]
    with pytest.raises(AssertionError):
        C.chunk_list_admit(idx, 1, 30, 30, 5)      # would overwrite the sink: a rebuild is due instead
    with pytest.raises(AssertionError):
        C.chunk_list_admit(idx, 1, 30, 29, 1)      # a chunk from before the rebuild is no new chunk


def test_chunk_list_admit_positions_follow_the_chunk_not_the_call():
    """Successive calls walk towards the sink (they do not start at the tail again), and admitting the
    same chunk again -- its later tokens arriving -- changes nothing."""
    idx = np.array([[0, 7, 3, 9, 5, 11]], dtype=np.int32)
    a = C.chunk_list_admit(idx, 1, 20, 20, 1)
    assert a.tolist() == [[0, 7, 3, 9, 5, 20]]
    b = C.chunk_list_admit(a, 1, 20, 20, 2)        # chunk 20 again (more of its tokens) and chunk 21
    assert b.tolist() == [[0, 7, 3, 9, 21, 20]]
    c = C.chunk_list_admit(b, 1, 20, 22, 2)
    assert c.tolist() == [[0, 7, 23, 22, 21, 20]]
    one_go = C.chunk_list_admit(idx, 1, 20, 20, 4)
    assert one_go.tolist() == c.tolist()


def test_chunk_list_admit_never_lists_a_chunk_twice():
    """The partly filled last chunk may already be listed when its next token arrives (the rebuild selected
    it): it moves to its position, the entry there takes its old place, nothing is evicted.  A duplicate
    would count twice in the softmax of the drafting pass."""
    idx = np.array([[0, 7, 12, 9, 5], [0, 2, 8, 4, 12], [12, 3, 8, 4, 6]], dtype=np.int32)
    out = C.chunk_list_admit(idx, 1, 12, 12, 1)
    assert out[0].tolist() == [0, 7, 5, 9, 12]     # traded places with the tail entry
    assert out[1].tolist() == [0, 2, 8, 4, 12]     # already at its position
    assert out[2].tolist() == [12, 3, 8, 4, 6]     # a sink entry stays where it is; nothing evicted
    for row in C.chunk_list_admit(idx, 1, 12, 12, 2):
        assert len(set(row.tolist())) == len(row)
    # the key set the list stands for: union of the old one and the new chunk, minus what was evicted
    before, after = set(idx[0].tolist()), set(out[0].tolist())
    assert after == before


def test_gather_then_dense_attention_equals_partial_attention():
    """The physical C_p and the in-place chunk list are the same key set (Alg. 1)."""
    rng = np.random.default_rng(2)
    hq, hkv, n, chunk = 4, 2, 300, 32
    q = rand_bits(rng, hq, D)
    k, v = rand_bits(rng, hkv, n, D), rand_bits(rng, hkv, n, D)
    idx = np.array([[0, 9, 4], [0, 2, 7]], dtype=np.int32)               # chunk 9 holds 12 tokens
    kg, vg = C.gather_chunks(k, v, idx, chunk)
    assert kg.shape == (hkv, 96, D)
    assert np.array_equal(kg[0, 32:44], k[0, 288:300]) and not kg[0, 44:64].any()   # zero-filled tail
    assert np.array_equal(vg[1, 64:96], v[1, 224:256])
    ref, _ = oracle.partial_attn(q, k, v, idx, chunk, 0.09)
    # dense attention over the gathered rows that are real tokens
    from helpers import dense_attention
    for h in range(hkv):
        valid = np.array([int(idx[h, j]) * chunk + w < n for j in range(3) for w in range(chunk)])
        out, _ = dense_attention(widen(q[h * 2:(h + 1) * 2]), widen(kg[h][valid]), widen(vg[h][valid]), 0.09)
        np.testing.assert_allclose(out, ref[h * 2:(h + 1) * 2], rtol=0, atol=1e-12)


@pytest.mark.parametrize("hq,hkv,n,chunk", [(4, 1, 130, 64), (12, 2, 257, 16), (8, 8, 64, 64), (6, 3, 100, 1)])
def test_key_sums_and_scores_reduce_to_the_definition_of_eq2(hq, hkv, n, chunk):
    rng = np.random.default_rng(3)
    q, k = rand_bits(rng, hq, D), rand_bits(rng, hkv, n, D)
    ks = C.chunk_key_sums(k, chunk)
    # sums against numpy's reduceat (a library routine), chunk by chunk
    starts = np.arange(0, n, chunk)
    np.testing.assert_allclose(ks, np.add.reduceat(widen(k), starts, axis=1), rtol=0, atol=1e-12)
    # scores from sums == the oracle of ts_chunk_scores (Eq. 2 written out token by token)
    s = C.scores_from_sums(ks, n, q, chunk, 0.0884)
    np.testing.assert_allclose(s, oracle.chunk_scores(q, k, chunk, 0.0884), rtol=0, atol=1e-10)


def test_key_sums_can_be_refreshed_incrementally():
    """Appending tokens changes only the sums of the chunks that received them."""
    rng = np.random.default_rng(4)
    k = rand_bits(rng, 2, 200, D)
    before = C.chunk_key_sums(k[:, :150], 64)      # chunks 0, 1, 2 (22 tokens in the last)
    after = C.chunk_key_sums(k, 64)                # chunks 0..3
    assert np.array_equal(before[:, :2], after[:, :2]) and not np.array_equal(before[:, 2], after[:, 2])
