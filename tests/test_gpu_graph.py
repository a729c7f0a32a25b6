"""The calls allocate nothing and never synchronise, so a whole layer-step can be captured into a HIP
graph.  The graph is replayed several times with the program's own eager work and synchronisations in
between, and every replay must reproduce the eager results bit for bit."""
import numpy as np
import pytest

import ts_synth as S

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("scored", [False, True])   # True: the verification pass leaves the scores (the benchmark's step)
@pytest.mark.parametrize("ci", [0, 1, 4])   # 4: 320 rows per KV head, the fp16 second product
def test_layer_step_in_a_graph_matches_eager(ci, scored):
    import torch
    import paper_2502_18890_amd as ts

    ts.load_library()
    cfg = S.CONFIGS[ci]
    dev = torch.device("cuda:0")
    x = S.make_layer_torch(cfg, 0, dev)
    hq, hkv, n, t = cfg.n_q_heads, cfg.n_kv_heads, cfg.n_tokens, cfg.n_tree
    ws_v = torch.empty(ts.workspace_bytes(ts.OP_TREE_VERIFY_SCORED, hq, hkv, n, t), dtype=torch.uint8, device=dev)
    ws_p = torch.empty(ts.workspace_bytes(ts.OP_PARTIAL_ATTN, hq, hkv, n, 0, cfg.n_sel, cfg.chunk), dtype=torch.uint8, device=dev)
    scores = torch.empty(hkv, cfg.n_chunks, dtype=torch.float32, device=dev)
    idx = torch.empty(hkv, cfg.n_sel, dtype=torch.int32, device=dev)
    out_p = torch.empty(hq, cfg.head_dim, dtype=torch.float32, device=dev)
    out_v = torch.empty(t, hq, cfg.head_dim, dtype=torch.float32, device=dev)

    def step():
        if scored:
            ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], cfg.scale,
                                out=out_v, workspace=ws_v, score_chunk=cfg.chunk, scores=scores)
        else:
            ts.chunk_scores(x["q"], x["k"], cfg.chunk, cfg.scale, out=scores)
        ts.topk_chunks(scores, cfg.n_sink, cfg.k, out=idx)
        ts.partial_kv_attn(x["q"], x["k"], x["v"], idx, cfg.chunk, cfg.scale, out=out_p, workspace=ws_p)
        if not scored:
            ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], cfg.scale,
                                out=out_v, workspace=ws_v)

    step()
    torch.cuda.synchronize()
    want = [scores.clone(), idx.clone(), out_p.clone(), out_v.clone()]

    side = torch.cuda.Stream()          # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                          # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()

    for rep in range(4):
        for buf in (scores, out_p, out_v):
            buf.fill_(float("nan"))     # eager work between the replays
        idx.fill_(-1)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref, name in zip((scores, idx, out_p, out_v), want, ("scores", "idx", "partial", "verify")):
            assert torch.equal(got, ref), "replay %d: %s differs from the eager result" % (rep, name)
