"""Benchmark of the decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

One step = one pass of the whole path over every layer's own cache of the workload, in the
order of the method's loop: tree verification over the full cache, which also leaves the chunk
scores (the query-key products of the tree's first token are the scores' terms, so the keys are
read once for both), top-k, partial-KV attention.  `--four-pass` times the step with the scores
as a pass of their own instead; either way the other step's time is reported beside it.  Caches
are resident in HBM before the timed region and each layer has its own, so every launch reads
cold data.  Prints one JSON line: `value` is microseconds per layer-step (one layer's cache);
`roofline` is the split kernel of the verification pass, its algorithmic bytes (K and V of the
cache and tree, queries, outputs) over its average duration from HIP events, against 8 TB/s;
`roofline_mfma` the same kernel's algorithmic flops; `cpu_baseline` the fp64 oracle timed on the
host cores over one layer's cache.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X published peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "verify_kernel_mha100k_pmc_traffic.txt")


def measured_traffic(workload_name):
    """HBM bytes per launch of the verify kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size), or None."""
    import re
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    m = re.search(r"^workload\s*=\s*(\S+)", text, re.M)
    t = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", text, re.M)
    if not m or not t or m.group(1) != workload_name:
        return None
    return int(t.group(1))


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=3, help="index into the workload list (3 = MHA, 100K tokens)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layer caches (0 = the config's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-loops", type=int, default=2, help="extra sweeps of the verify kernel alone for the roofline figure")
    ap.add_argument("--four-pass", action="store_true",
                    help="time the step with the chunk scores as a pass of their own (ts_chunk_scores) instead of "
                         "leaving them to the verification pass (ts_tree_verify_attn_scored)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one whole step (all layers) in a HIP graph and time its replays instead of eager launches")
    ap.add_argument("--hold", type=float, default=0.0,
                    help="utility mode: repeat the verification pass alone for this many seconds and exit, so that an "
                         "external tool (rocm-smi --showclocks) can sample the clock the kernel runs at")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run an elementwise kernel that reads 1 GiB and writes 1 GiB (to scale rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def cpu_baseline(cfg, layer_inputs, budget_s=12.0):
    """Time the fp64 oracle (as it stands, untuned) on whole layer-steps of the workload -- one
    layer's cache, whole path, repeated until about budget_s seconds of CPU work are done."""
    import numpy as np
    import oracle
    import ts_synth as S

    bits = lambda t: S.torch_bf16_to_bits(t)
    q, k, v = bits(layer_inputs["q"]), bits(layer_inputs["k"]), bits(layer_inputs["v"])
    q_tree, k_tree, v_tree = bits(layer_inputs["q_tree"]), bits(layer_inputs["k_tree"]), bits(layer_inputs["v_tree"])
    reps, dt = 0, 0.0
    t0 = time.perf_counter()
    while True:
        sc = oracle.chunk_scores(q, k, cfg.chunk, cfg.scale)
        idx = oracle.topk_chunks(sc.astype(np.float32), cfg.n_sink, cfg.k)
        oracle.partial_attn(q, k, v, idx, cfg.chunk, cfg.scale)
        oracle.tree_verify(q_tree, k, v, k_tree, v_tree, layer_inputs["parent"], cfg.scale)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= 64:
            break
    return {"value": round(dt * 1e6 / reps, 1), "unit": "us/layer-step", "cores": oracle.num_threads(),
            "kind": "oracle", "seconds_measured": round(dt, 2),
            "sample": "fp64 oracle (OpenMP over heads/rows), whole path (scores, top-k, partial attention, tree-verify) "
                      "on one layer's cache of the workload, all %d KV heads, %d repetitions" % (cfg.n_kv_heads, reps)}


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (got --gpus %d); nothing here uses a second GPU" % args.gpus)
    import torch
    import paper_2502_18890_amd as ts
    import ts_synth as S

    ts.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = S.CONFIGS[args.config]
    n_layers = args.layers or cfg.n_layers
    layer_bytes = cfg.n_kv_heads * cfg.n_tokens * cfg.head_dim * 2 * 2
    # small configs: replicate until the rotating working set is well beyond the on-die caches
    while n_layers * layer_bytes < (2 << 30):
        n_layers += cfg.n_layers

    layers = [S.make_layer_torch(cfg, l, dev) for l in range(n_layers)]
    hq, hkv, n, t = cfg.n_q_heads, cfg.n_kv_heads, cfg.n_tokens, cfg.n_tree
    ws_v = torch.empty(ts.workspace_bytes(ts.OP_TREE_VERIFY, hq, hkv, n, t), dtype=torch.uint8, device=dev)
    ws_vs = torch.empty(ts.workspace_bytes(ts.OP_TREE_VERIFY_SCORED, hq, hkv, n, t), dtype=torch.uint8, device=dev)
    ws_p = torch.empty(ts.workspace_bytes(ts.OP_PARTIAL_ATTN, hq, hkv, n, 0, cfg.n_sel, cfg.chunk), dtype=torch.uint8, device=dev)
    scores = torch.empty(hkv, cfg.n_chunks, dtype=torch.float32, device=dev)
    idx = torch.empty(hkv, cfg.n_sel, dtype=torch.int32, device=dev)
    out_p = torch.empty(hq, cfg.head_dim, dtype=torch.float32, device=dev)
    out_v = torch.empty(t, hq, cfg.head_dim, dtype=torch.float32, device=dev)
    torch.cuda.synchronize()

    def do_scores(x):
        ts.chunk_scores(x["q"], x["k"], cfg.chunk, cfg.scale, out=scores)

    def do_topk(x):
        ts.topk_chunks(scores, cfg.n_sink, cfg.k, out=idx)

    def do_partial(x):
        ts.partial_kv_attn(x["q"], x["k"], x["v"], idx, cfg.chunk, cfg.scale, out=out_p, workspace=ws_p)

    def do_verify(x):
        ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], cfg.scale,
                            out=out_v, workspace=ws_v)

    def do_verify_scored(x):
        # the verification pass also leaves the chunk scores for the query of tree node 0 (= x["q"] in these inputs)
        ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], cfg.scale,
                            out=out_v, workspace=ws_vs, score_chunk=cfg.chunk, scores=scores)

    def step_four_pass():
        for x in layers:
            do_scores(x)
            do_topk(x)
            do_partial(x)
            do_verify(x)

    def step_scored():
        # the order of Alg. 1: verification over the full cache (whose query-key products give the scores),
        # rebuild of the partial cache's chunk list, drafting pass over it
        for x in layers:
            do_verify_scored(x)
            do_topk(x)
            do_partial(x)

    step = step_four_pass if args.four_pass else step_scored
    do_verify_timed = do_verify if args.four_pass else do_verify_scored

    def timed(fn, reps):
        """ms per call of fn over reps calls, HIP events on the current stream."""
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    for _ in range(args.warmup):
        step()
    (step_scored if args.four_pass else step_four_pass)()   # the other step, timed after the K steps for comparison
    torch.cuda.synchronize()
    # both ways of getting the scores select the same chunks (same query, same keys; sums in another order)
    x0 = layers[0]
    do_scores(x0); do_topk(x0)
    idx_a = idx.clone()
    do_verify_scored(x0); do_topk(x0)
    same_sets = sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(idx_a.cpu(), idx.cpu())) / float(idx.numel())
    assert same_sets > 0.98, "scores from the verification pass select other chunks than the scoring pass (%.3f)" % same_sets
    if args.hold > 0:
        t_start, calls = time.time(), 0
        while time.time() - t_start < args.hold:
            for x in layers:
                do_verify(x)
            torch.cuda.synchronize()
            calls += len(layers)
        print("bench.py --hold: %s, %d verification passes in %.1f s, %.1f us each"
              % (cfg.name, calls, time.time() - t_start, (time.time() - t_start) / calls * 1e6), flush=True)
        return
    run_step = step
    if args.graph:   # the calls allocate nothing and never synchronise, so a step can be captured as it is
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        torch.cuda.synchronize()
        run_step = graph.replay
        run_step()
        torch.cuda.synchronize()
    wall0 = time.perf_counter()
    ms_per_step = timed(run_step, args.steps)
    wall = time.perf_counter() - wall0
    other_step = step_scored if args.four_pass else step_four_pass
    ms_other = timed(other_step, max(2, args.steps // 4))

    # per-function breakdown (each swept over all layers, same rotation)
    def sweep(fn):
        return lambda: [fn(x) for x in layers]
    reps = max(2, args.steps // 4)

    def spread(fn, n_sweeps):
        """us per layer of fn, each sweep over the layers timed on its own: mean, median, p10, p90."""
        evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_sweeps + 1)]
        torch.cuda.synchronize()
        evs[0].record()
        for i in range(n_sweeps):
            for x in layers:
                fn(x)
            evs[i + 1].record()
        torch.cuda.synchronize()
        us = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 / n_layers for i in range(n_sweeps))
        pick = lambda q: us[min(len(us) - 1, int(round(q * (len(us) - 1))))]
        return {"mean": sum(us) / len(us), "median": pick(0.5), "p10": pick(0.1), "p90": pick(0.9)}

    stats = {name: spread(fn, max(reps, 10))
             for name, fn in (("scores", do_scores), ("topk", do_topk), ("partial", do_partial), ("verify", do_verify),
                              ("verify_scored", do_verify_scored))}
    parts = {name: st["mean"] for name, st in stats.items()}

    # cache-maintenance calls around the path (not part of `value`): incremental key sums make
    # the scoring pass read n_chunks*128 floats instead of every key
    ksum = [ts.chunk_key_sums(x["k"], cfg.chunk) for x in layers]
    kg, vg = ts.gather_chunks(layers[0]["k"], layers[0]["v"], idx, cfg.chunk)
    acc = list(range(min(4, t)))
    extras = {
        "scores_from_key_sums": lambda i, x: ts.chunk_scores_from_sums(ksum[i], n, x["q"], cfg.chunk, cfg.scale, out=scores),
        "key_sums_full_rebuild": lambda i, x: ts.chunk_key_sums(x["k"], cfg.chunk, out=ksum[i]),
        "key_sums_last_chunk": lambda i, x: ts.chunk_key_sums(x["k"], cfg.chunk, out=ksum[i], chunk_begin=cfg.n_chunks - 1),
        "append_accepted_4": lambda i, x: ts.append_accepted(x["k"], x["v"], n - len(acc), x["k_tree"], x["v_tree"], acc),
        "chunk_list_admit_1": lambda i, x: ts.chunk_list_admit(idx, cfg.n_sink, cfg.n_chunks - 1, cfg.n_chunks - 1, 1),
        "gather_chunks": lambda i, x: ts.gather_chunks(x["k"], x["v"], idx, cfg.chunk),
    }
    do_topk(layers[0])
    maint = {}
    for name, fn in extras.items():
        if name == "append_accepted_4":
            saved = [(x["k"][:, n - len(acc):].clone(), x["v"][:, n - len(acc):].clone()) for x in layers]
        maint[name] = timed(lambda: [fn(i, x) for i, x in enumerate(layers)], reps) * 1e3 / n_layers
        if name == "append_accepted_4":      # put the overwritten cache rows back
            for x, (sk, sv) in zip(layers, saved):
                x["k"][:, n - len(acc):] = sk
                x["v"][:, n - len(acc):] = sv
    del kg, vg, ksum

    # penalized probabilities + pool sampling for the T verification rows (once per step, not per
    # layer; not part of `value`): vocabulary of the model the workload is shaped like
    vocab = {"tiny": 32000, "qwen2.5-1.5b": 151936, "llama3.1-8b": 128256, "yarn-llama2-7b-mha": 32000,
             "qwen2.5-14b": 152064}.get(cfg.name, 32000)
    gen = torch.Generator(device=dev)
    gen.manual_seed(cfg.seed)
    logits = torch.randn(t, vocab, generator=gen, device=dev, dtype=torch.float32) * 3.0
    window = torch.randint(0, vocab, (1024,), generator=gen, device=dev, dtype=torch.int32)
    uni = torch.rand(t, generator=gen, device=dev, dtype=torch.float32)
    probs = torch.empty_like(logits)
    ws_s = torch.empty(max(1, ts.load_library().ts_sampling_workspace_bytes(t, vocab)), dtype=torch.uint8, device=dev)
    sampling = {
        "penalized_probs": timed(lambda: ts.penalized_probs(logits, window, 1.0, 1.15, out=probs, workspace=ws_s), 20) * 1e3,
        "sample_min_p": timed(lambda: ts.sample_tokens(probs, ts.SAMPLE_MIN_P, 0.1, uni), 20) * 1e3,
        "sample_top_p": timed(lambda: ts.sample_tokens(probs, ts.SAMPLE_TOP_P, 0.9, uni), 20) * 1e3,
    }
    sampling_bytes = 3 * t * vocab * 4   # logits read twice, probabilities written once
    del logits, probs

    # the dominant kernel alone (split kernel of the verification pass), for the roofline
    ts.tune_set("verify_stage", 1)
    try:
        timed(sweep(do_verify_timed), 1)
        kern_us = timed(sweep(do_verify_timed), max(1, args.kernel_loops)) * 1e3 / n_layers
    finally:
        ts.tune_set("verify_stage", 0)
    # what plain reading of the same cache buffers sustains (nothing but loads): the practical ceiling
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_bytes = 0
    def do_probe(x):
        ts.stream_read_probe(x["k"], sink)
        ts.stream_read_probe(x["v"], sink)
    if all(x["k"].is_contiguous() and x["v"].is_contiguous() for x in layers):
        probe_bytes = 2 * layers[0]["k"].numel() * 2
        timed(sweep(do_probe), 1)
        probe_us = timed(sweep(do_probe), max(1, args.kernel_loops)) * 1e3 / n_layers
    alg_bytes = (hkv * n * cfg.head_dim * 2 * 2 + t * hkv * cfg.head_dim * 2 * 2 + t * hq * cfg.head_dim * 2
                 + t * hq * cfg.head_dim * 4)
    achieved = alg_bytes / (kern_us * 1e-6) / 1e9
    # the same launch against the matrix-core roofline: algorithmic flops = QK^T and PV once each,
    # 4*g*T*d flops per cached or tree key and KV head (the second, low-order PV product that keeps
    # the weights' precision is an implementation cost and is not counted)
    alg_flops = 4.0 * cfg.group * t * cfg.head_dim * (n + t) * hkv
    kernel_name = "verify_dma_kernel (16x16x32 MFMA)" if cfg.group * t <= 32 else "verify_wide_kernel (32x32x16 MFMA)"

    us_per_layer_step = ms_per_step * 1e3 / n_layers
    # beyond 128 query rows per KV head the verification pass multiplies fp16 weights with fp16 values
    dtype = "bf16 inputs, fp32 accumulate" if cfg.group * t <= 128 else "bf16 inputs, fp32 accumulate (weights x values of the verification pass in fp16)"
    res = {
        "metric": "us per layer-step: chunk scores + top-k + partial-KV attention + tree-verify attention over the full cache",
        "value": round(us_per_layer_step, 3), "unit": "us/layer-step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s: %d q heads / %d kv heads, d=128, N=%d cached tokens, chunk %d, top-k %d+%d chunks, tree %d nodes, %d layer caches, batch 1" % (
            cfg.name, hq, hkv, n, cfg.chunk, cfg.k, cfg.n_sink, t, n_layers), "config_index": args.config,
            "layers": n_layers, "n_tokens": n, "launch": "hip graph replay" if args.graph else "eager"},
        "step": ("four passes: ts_chunk_scores, ts_topk_chunks, ts_partial_kv_attn, ts_tree_verify_attn" if args.four_pass else
                 "three passes: ts_tree_verify_attn_scored (verification; its query-key products of tree node 0 also give the "
                 "chunk scores, same values as ts_chunk_scores for that query), ts_topk_chunks, ts_partial_kv_attn"),
        "other_step_us_per_layer": {("scores_left_to_verification" if args.four_pass else "four_passes"): round(ms_other * 1e3 / n_layers, 3)},
        "breakdown_us_per_layer": {k: round(v, 3) for k, v in parts.items()},
        "breakdown_spread_us_per_layer": {k: {q: round(v, 3) for q, v in st.items() if q != "mean"} for k, st in stats.items()},
        "verify_plus_partial_us_per_layer": round(parts["verify"] + parts["partial"], 3),
        # Alg. 1 rebuilds the partial cache once per |B| - |S| = k * chunk accepted tokens: the scoring pass and the
        # selection, spread over those tokens (what they cost when they are passes of their own)
        "rebuild_amortised": {"scores_plus_topk_us_per_layer": round(parts["scores"] + parts["topk"], 3),
                              "tokens_between_rebuilds": cfg.k * cfg.chunk,
                              "us_per_layer_per_accepted_token": round((parts["scores"] + parts["topk"]) / (cfg.k * cfg.chunk), 5)},
        "cache_maintenance_us_per_layer": {k: round(v, 3) for k, v in maint.items()},
        "sampling_us_per_step": dict({k: round(v, 3) for k, v in sampling.items()}, rows=t, vocab=vocab, window=1024,
                                     penalized_probs_gbs=round(sampling_bytes / (sampling["penalized_probs"] * 1e-6) / 1e9, 1)),
        "verify_call_gbs": round(alg_bytes / (parts["verify"] * 1e-6) / 1e9, 1),
        "wall_s_timed_region": round(wall, 3),
        "roofline": {"kernel": kernel_name + ", split kernel of the tree-verify pass", "bound": "hbm",
                     "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(achieved / HBM_PEAK_GBS, 4),
                     "traffic": measured_traffic(cfg.name) if n == cfg.n_tokens else None,
                     "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": round(kern_us, 3)},
        "stream_read_ceiling": ({"GBps": round(probe_bytes / (probe_us * 1e-6) / 1e9, 1), "bytes_per_layer": probe_bytes,
                                 "us_per_layer": round(probe_us, 3),
                                 "frac_of_peak": round(probe_bytes / (probe_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                 "roofline_kernel_frac_of_ceiling": round(achieved / (probe_bytes / (probe_us * 1e-6) / 1e9), 4),
                                 "what": "a kernel of nothing but 128-bit loads over the same K and V buffers, same rotation"}
                                if probe_bytes else None),
        "roofline_mfma": {"bound": "mfma", "achieved": round(alg_flops / (kern_us * 1e-6) / 1e12, 2), "peak": 2500.0,
                          "unit": "TFLOP/s", "frac": round(alg_flops / (kern_us * 1e-6) / 2.5e15, 4),
                          "algorithmic_flops_per_launch": alg_flops, "flops_per_byte": round(alg_flops / alg_bytes, 1)},
    }
    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, layers[0])
    print(json.dumps(res))


if __name__ == "__main__":
    main()
