"""GPU parity at the full benchmark sizes, in the launch configuration bench.py times: one
layer of each large workload is generated on the device, the whole path runs through the C ABI,
and the fp64 oracle checks every chunk score (from the scoring pass and from the verification pass that
leaves them), the selection (bit-exact from the GPU's scores),
the whole partial-attention output, and a sample of tree-verification rows it computes one by one."""
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
    # tree verification: sampled rows, always including the corners
    rng = np.random.default_rng(cfg.seed)
    rows = {(0, 0), (cfg.n_tree - 1, cfg.n_q_heads - 1), (0, cfg.n_q_heads - 1), (cfg.n_tree - 1, 0)}
    while len(rows) < 24:
        rows.add((int(rng.integers(cfg.n_tree)), int(rng.integers(cfg.n_q_heads))))
    rows = sorted(rows)
    ref_v, ref_lse_v = oracle.tree_verify(bits(x["q_tree"]), k, v, bits(x["k_tree"]), bits(x["v_tree"]), x["parent"],
                                          cfg.scale, rows=rows)
    got_v = out_v.cpu().numpy()[[r[0] for r in rows], [r[1] for r in rows]]
    got_lse = lse_v.cpu().numpy()[[r[0] for r in rows], [r[1] for r in rows]]
    assert_close(got_v, ref_v, "verify rows cfg%d" % ci)
    assert_close(got_lse, ref_lse_v, "verify lse cfg%d" % ci)
    # a property that holds at any size: everything finite
    assert torch.isfinite(out_v).all() and torch.isfinite(lse_v).all()
