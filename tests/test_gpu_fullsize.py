"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: one
layer of each large workload is generated on the device, the whole path runs through the C ABI,
and the fp64 oracle checks every chunk score (from the scoring pass and from the verification pass that
leaves them), the selection (bit-exact from the GPU's scores),
the whole partial-attention output, and every row of the tree verification (output and lse).  One more case runs
the verification alone at the paper's own width: the 40-node [1,3,3,3] tree plus 20 retrieved 4-grams that share its
root (Sec. 3.2 "Token Reutilization", App. E; 100 tokens) over the 100000-token MHA layer, and over the 65536-token
layer of the 4-way GQA shape (400 query rows per KV head)."""
import numpy as np
import pytest

import oracle
import ts_synth as S
from gpu_util import assert_close

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("ci", [2, 3, 4])
def test_full_size_layer(ci):
    import torch
    import paper_2502_18890_amd as ts

    cfg = S.CONFIGS[ci]
    dev = torch.device("cuda:0")
    x = S.make_layer_torch(cfg, 0, dev)
    sc = ts.chunk_scores(x["q"], x["k"], cfg.chunk, cfg.scale)
    idx = ts.topk_chunks(sc, cfg.n_sink, cfg.k)
    out_p, lse_p = ts.partial_kv_attn(x["q"], x["k"], x["v"], idx, cfg.chunk, cfg.scale, want_lse=True)
    out_v, lse_v = ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], cfg.scale,
                                       want_lse=True)
    # the call the benchmark's step uses: verification that also leaves the chunk scores (tree node 0 carries q)
    out_s, lse_s, sc_s = ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], cfg.scale,
                                             want_lse=True, score_chunk=cfg.chunk)
    torch.cuda.synchronize()
    assert torch.equal(out_s, out_v) and torch.equal(lse_s, lse_v)

    bits = S.torch_bf16_to_bits
    q, k, v = bits(x["q"]), bits(x["k"]), bits(x["v"])
    # chunk scores: all of them
    ref_sc = oracle.chunk_scores(q, k, cfg.chunk, cfg.scale)
    assert_close(sc.cpu().numpy(), ref_sc, "scores cfg%d" % ci)
    assert_close(sc_s.cpu().numpy(), ref_sc, "scores from the verification pass cfg%d" % ci)
    idx_s = ts.topk_chunks(sc_s, cfg.n_sink, cfg.k).cpu().numpy()
    np.testing.assert_array_equal(idx_s, oracle.topk_chunks(sc_s.cpu().numpy(), cfg.n_sink, cfg.k))
    # selection: bit-exact from the same fp32 score vector
    idx_h = idx.cpu().numpy()
    np.testing.assert_array_equal(idx_h, oracle.topk_chunks(sc.cpu().numpy(), cfg.n_sink, cfg.k))
    assert idx_h.shape == (cfg.n_kv_heads, cfg.n_sel) and np.all(idx_h[:, 0] == 0)
    # planted chunks (where the workload has them) are mostly recovered
    if x["planted"].shape[1] > 0:
        hits = [len(set(x["planted"][h].tolist()) & set(idx_h[h].tolist())) for h in range(cfg.n_kv_heads)]
        assert np.mean(hits) >= 0.6 * min(x["planted"].shape[1], cfg.k)
    # partial attention: every output
    ref_p, ref_lse_p = oracle.partial_attn(q, k, v, idx_h, cfg.chunk, cfg.scale)
    assert_close(out_p.cpu().numpy(), ref_p, "partial out cfg%d" % ci)
    assert_close(lse_p.cpu().numpy(), ref_lse_p, "partial lse cfg%d" % ci)
    # tree verification: every row (node, head) of out and lse
    ref_v, ref_lse_v = oracle.tree_verify(bits(x["q_tree"]), k, v, bits(x["k_tree"]), bits(x["v_tree"]), x["parent"],
                                          cfg.scale)
    assert_close(out_v.cpu().numpy(), ref_v, "verify out cfg%d" % ci)
    assert_close(lse_v.cpu().numpy(), ref_lse_v, "verify lse cfg%d" % ci)
    # the bar also holds row by row: no single (node, head) row hides behind the others' norm
    got = out_v.cpu().numpy().astype(np.float64)
    row_rel = np.linalg.norm(got - ref_v, axis=-1) / np.linalg.norm(ref_v, axis=-1)
    assert float(row_rel.max()) <= 1e-3, ("worst row", np.unravel_index(int(row_rel.argmax()), row_rel.shape), float(row_rel.max()))


def paper_width_tree():
    """Parent array of the widest verification input the paper runs: the [1,3,3,3] tree (1 + 3 + 9 + 27 = 40 nodes)
    followed by 20 retrieved 4-grams whose first token is the root, i.e. 20 chains of 3 below node 0."""
    parent = [-1] + [0] * 3 + [1 + i // 3 for i in range(9)] + [4 + i // 3 for i in range(27)]
    for _ in range(20):
        b = len(parent)
        parent += [0, b, b + 1]
    return np.asarray(parent, dtype=np.int32)


@pytest.mark.parametrize("ci", [3, 2])
def test_full_size_paper_width_verification(ci):
    """The paper's widest verification input (Sec. 3.2: the 40-node tree plus 20 retrieved 4-grams, 100 tokens) over a full
    cache: 100 query rows per KV head on the MHA shape, 400 on the 4-way GQA shape (two row tiles)."""
    import torch
    import paper_2502_18890_amd as ts

    cfg = S.CONFIGS[ci]
    parent = paper_width_tree()
    t = len(parent)
    assert t == 100
    dev = torch.device("cuda:0")
    x = S.make_layer_torch(cfg, 1, dev, n_tree=t)
    out_v, lse_v = ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], parent, cfg.scale, want_lse=True)
    out_s, lse_s, sc_s = ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], parent, cfg.scale,
                                             want_lse=True, score_chunk=cfg.chunk)
    torch.cuda.synchronize()
    assert torch.equal(out_s, out_v) and torch.equal(lse_s, lse_v)
    bits = S.torch_bf16_to_bits
    k, v = bits(x["k"]), bits(x["v"])
    ref_v, ref_lse_v = oracle.tree_verify(bits(x["q_tree"]), k, v, bits(x["k_tree"]), bits(x["v_tree"]), parent, cfg.scale)
    assert_close(out_v.cpu().numpy(), ref_v, "verify out, 100 tree tokens x %d cached" % cfg.n_tokens)
    assert_close(lse_v.cpu().numpy(), ref_lse_v, "verify lse, 100 tree tokens x %d cached" % cfg.n_tokens)
    assert_close(sc_s.cpu().numpy(), oracle.chunk_scores(bits(x["q_tree"])[0], k, cfg.chunk, cfg.scale), "scores left by it")
