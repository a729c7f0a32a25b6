"""The calls in the order of the method's loop (Alg. 1), several iterations on one growing cache:
drafting attention over the partial cache, verification over the full cache (which also leaves the
chunk scores), acceptance of a path of the tree, append to the full cache, and either the rebuild of
the partial cache's chunk list (when the new tokens' chunks would reach the sink entries) or the
admission of the chunks that received tokens, each from its first token on, so that the next drafting
pass sees every generated token.  The fp64 oracle does the same on host copies; every output of every
iteration is compared (rows and indices byte-exact, floating point to the bar).  Besides, the drafting
output is checked against plain dense attention over the duplicate-free union of the listed chunks'
tokens, which must contain every token generated since the rebuild: a chunk listed twice, or a new
token the list does not cover, fails there even if the oracle mirrored the same mistake."""
import math

import numpy as np
import pytest

import oracle
import ts_synth as S
from oracle import cache_ops as C
from gpu_util import assert_close, dev
from helpers import dense_attention, rand_bits, widen

pytestmark = pytest.mark.gpu
D = 128
SCALE = 1.0 / math.sqrt(D)


def _path_to(parent, node):
    path = []
    while node >= 0:
        path.append(int(node))
        node = parent[node]
    return path[::-1]


@pytest.mark.parametrize("hq,hkv,chunk,n_sink,k_sel,n0,t,iters", [(8, 2, 32, 1, 2, 700, 12, 14), (4, 4, 64, 1, 1, 375, 7, 14),
                                                                  (12, 2, 32, 2, 1, 1500, 20, 10), (4, 2, 32, 1, 6, 200, 6, 8)])
def test_generation_loop_calls_compose(hq, hkv, chunk, n_sink, k_sel, n0, t, iters):
    import torch
    import paper_2502_18890_amd as ts
    ts.load_library()
    rng = np.random.default_rng(1000 + hq + n0)
    cap = n0 + iters * t + chunk
    k_h, v_h = rand_bits(rng, hkv, cap, D), rand_bits(rng, hkv, cap, D)      # host mirror (bf16 bits)
    k_d, v_d = dev(k_h), dev(v_h)
    n = n0
    budget, sink_tokens = (n_sink + k_sel) * chunk, n_sink * chunk

    # prefill: the chunk list from the scoring pass proper
    q = rand_bits(rng, hq, D)
    sc = ts.chunk_scores(dev(q), k_d[:, :n], chunk, SCALE)
    idx_d = ts.topk_chunks(sc, n_sink, k_sel)
    idx_h = oracle.topk_chunks(sc.cpu().numpy(), n_sink, k_sel)
    np.testing.assert_array_equal(idx_d.cpu().numpy(), idx_h)
    n_at_rebuild = n
    rebuilds = admits = relisted = by_rebuild = 0

    def check_list_and_draft(q, out_p, it):
        """No chunk twice; every token generated since the rebuild is covered; the drafting output equals
        dense attention over the union of the listed chunks' tokens (each token once)."""
        g = hq // hkv
        for h in range(hkv):
            ids = idx_h[h].tolist()
            assert len(set(ids)) == len(ids), ("chunk listed twice", it, h, ids)
            assert ids[:n_sink] == list(range(n_sink))
            toks = sorted({tk for c in ids for tk in range(c * chunk, min(n, (c + 1) * chunk))})
            assert set(range(n_at_rebuild, n)) <= set(toks), ("generated token not visible to the draft", it, h)
            ref, _ = dense_attention(widen(q[h * g:(h + 1) * g]), widen(k_h[h, toks]), widen(v_h[h, toks]), SCALE)
            assert_close(out_p[h * g:(h + 1) * g], ref, "draft vs dense attention over the union, it=%d head %d" % (it, h))

    for it in range(iters):
        q = rand_bits(rng, hq, D)
        # drafting pass over the partial cache
        out_p = ts.partial_kv_attn(dev(q), k_d[:, :n], v_d[:, :n], idx_d, chunk, SCALE)
        assert_close(out_p.cpu().numpy(), oracle.partial_attn(q, k_h[:, :n], v_h[:, :n], idx_h, chunk, SCALE)[0], "draft it=%d" % it)
        check_list_and_draft(q, out_p.cpu().numpy(), it)
        # verification of a tree rooted at the same token over the full cache; it leaves the scores
        q_tree = rand_bits(rng, t, hq, D)
        q_tree[0] = q
        k_tree, v_tree = rand_bits(rng, t, hkv, D), rand_bits(rng, t, hkv, D)
        parent = np.full(t, -1, dtype=np.int32)
        for i in range(1, t):                       # one tree, rooted at node 0, with some long branches
            parent[i] = i - 1 if rng.random() < 0.6 else rng.integers(0, i)
        out_v, sc = ts.tree_verify_attn(dev(q_tree), k_d[:, :n], v_d[:, :n], dev(k_tree), dev(v_tree), parent, SCALE,
                                        score_chunk=chunk)
        assert_close(out_v.cpu().numpy(), oracle.tree_verify(q_tree, k_h[:, :n], v_h[:, :n], k_tree, v_tree, parent, SCALE)[0],
                     "verify it=%d" % it)
        assert_close(sc.cpu().numpy(), oracle.chunk_scores(q, k_h[:, :n], chunk, SCALE), "scores it=%d" % it)
        # accept a root-to-node path and append it
        accepted = max((_path_to(parent, int(c)) for c in rng.integers(0, t, size=3)), key=len)
        new_n = ts.append_accepted(k_d, v_d, n, dev(k_tree), dev(v_tree), accepted)
        k_h, v_h = C.append_accepted(k_h, v_h, n, k_tree, v_tree, accepted)
        assert new_n == n + len(accepted)
        np.testing.assert_array_equal(S.torch_bf16_to_bits(k_d[:, :new_n]), k_h[:, :new_n])
        np.testing.assert_array_equal(S.torch_bf16_to_bits(v_d[:, :new_n]), v_h[:, :new_n])
        # partial cache: rebuild when the new tokens' chunks would reach the sink entries (the rebuild trigger of
        # Alg. 1 with the size at the last rebuild rounded down to a chunk boundary), else admit the chunks that
        # received tokens -- the first of them possibly for the second time, or already listed by the rebuild
        base = n_at_rebuild // chunk
        due = ts.refresh_due(new_n, base * chunk, budget, sink_tokens)
        assert due == C.refresh_due(new_n, base * chunk, budget, sink_tokens)
        assert due == ((new_n - 1) // chunk - base + 1 > k_sel)
        if due:
            sc = ts.chunk_scores(dev(q), k_d[:, :new_n], chunk, SCALE)
            idx_d = ts.topk_chunks(sc, n_sink, k_sel)
            idx_h = oracle.topk_chunks(sc.cpu().numpy(), n_sink, k_sel)
            n_at_rebuild = new_n
            rebuilds += 1
        else:
            first_new, n_new = n // chunk, (new_n - 1) // chunk - n // chunk + 1
            listed = any(first_new in idx_h[h, n_sink:].tolist() for h in range(hkv))
            relisted += int(listed)
            by_rebuild += int(listed and n == n_at_rebuild)     # the selection itself had listed the partly filled last chunk
            ts.chunk_list_admit(idx_d, n_sink, base, first_new, n_new)
            idx_h = C.chunk_list_admit(idx_h, n_sink, base, first_new, n_new)
            admits += 1
        np.testing.assert_array_equal(idx_d.cpu().numpy(), idx_h)
        n = new_n
    torch.cuda.synchronize()
    print("loop: %d tokens appended, %d rebuilds, %d admissions, %d of a chunk some head already listed (%d times by the selection)"
          % (n - n0, rebuilds, admits, relisted, by_rebuild))
    assert n > n0 and admits > 0 and relisted > 0 and (rebuilds > 0 or by_rebuild > 0)
