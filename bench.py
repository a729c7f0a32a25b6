"""Benchmark of the decode-attention hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3]

One step = one pass of the whole path over every layer's own cache of the workload, in the
order of the method's loop: tree verification over the full cache, which also leaves the chunk
scores (the query-key products of the tree's first token are the scores' terms, so the keys are
read once for both), top-k, partial-KV attention.  That step rests on a reading (the query that
ranks the cache is tree node 0's, in the verification pass); the step with the scores as a pass of
their own (ts_chunk_scores, any query) is timed beside it and reported as `value_no_reading`.
`--four-pass` makes that one `value`.  Caches are resident in HBM before the timed region and each
layer has its own, so every launch reads cold data.  Prints one JSON line: `value` is microseconds
per layer-step (one layer's cache); `roofline` is the split kernel of the verification pass, its
algorithmic bytes (K and V of the cache and tree, queries, outputs) over its average duration from
HIP events, against 8 TB/s; `roofline_mfma` the same kernel's algorithmic flops; `cpu_baseline` the
fp64 oracle timed on the host cores over one layer's cache, with all threads and with one.

After the headline workload the default run also times the other large workloads and the paper's
own verification width on the headline cache (`workloads`), each with its step, its verification
kernel alone and that kernel's fraction of both rooflines, and the two small workloads eager and as
a HIP graph replay (`small_workloads`).  `--config i` alone skips those.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published peak
MFMA_PEAK_TFLOPS = 2500.0  # dense bf16 / fp16
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "verify_kernel_mha100k_pmc_traffic.txt")
HEADLINE = 3


def measured_traffic(workload_name, library_version):
    """HBM bytes per launch of the verify kernel from the committed rocprofv3 --pmc summary
    (FETCH_SIZE + WRITE_SIZE, scaled by a copy kernel of known size), or None when there is none for this
    workload or it was taken with another version of the library (the kernels may have changed since)."""
    import re
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    m = re.search(r"^workload\s*=\s*(\S+)", text, re.M)
    t = re.search(r"^traffic_bytes_per_launch\s*=\s*(\d+)", text, re.M)
    ver = re.search(r"^library_version\s*=\s*(\d+)", text, re.M)
    if not m or not t or not ver or m.group(1) != workload_name or int(ver.group(1)) != library_version:
        return None
    return int(t.group(1))


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=None,
                    help="index into the workload list; default: 3 (MHA, 100K tokens) as the headline, then the others in brief")
    ap.add_argument("--tree", type=int, default=0, help="override the number of tree nodes (100 = the paper's widest verification input)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layer caches (0 = the config's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernel-loops", type=int, default=2, help="extra sweeps of the verify kernel alone for the roofline figure")
    ap.add_argument("--four-pass", action="store_true",
                    help="make the step with the chunk scores as a pass of their own (ts_chunk_scores) the reported `value`")
    ap.add_argument("--graph", action="store_true",
                    help="capture one whole step (all layers) in a HIP graph and time its replays instead of eager launches")
    ap.add_argument("--hold", type=float, default=0.0,
                    help="utility mode: repeat the verification pass alone for this many seconds and exit, so that an "
                         "external tool (rocm-smi --showclocks --showpower) can sample the chip while the kernel runs")
    ap.add_argument("--hold-what", choices=("verify", "stream-read"), default="verify",
                    help="what --hold repeats: the verification pass, or the kernel of nothing but loads over the same K and V buffers")
    ap.add_argument("--zero-cache", action="store_true",
                    help="utility: fill every layer's K and V with zeros before timing (same instructions, same bytes moved, "
                         "fewer bits toggling in the multipliers: shows how much of a pass's time is set by power)")
    ap.add_argument("--splits", type=int, default=0,
                    help="utility: force the number of cache splits per KV head of the verification pass (0 = the library's choice); "
                         "fewer splits than the chip has room for leave compute units idle, which shows what the pass does per "
                         "compute unit when the chip's power limit is out of the way")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run an elementwise kernel that reads 1 GiB and writes 1 GiB (to scale rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    return ap.parse_args()


def paper_width_tree():
    """The widest verification input of the paper (Sec. 3.2 "Token Reutilization", App. E): the [1,3,3,3] tree of
    40 nodes plus 20 retrieved 4-grams that share its root, i.e. 20 chains of 3 below node 0: 100 tokens."""
    parent = [-1] + [0] * 3 + [1 + i // 3 for i in range(9)] + [4 + i // 3 for i in range(27)]
    for _ in range(20):
        b = len(parent)
        parent += [0, b, b + 1]
    return parent


def cpu_baseline(cfg, x, budget_s=8.0):
    """Time the fp64 oracle (as it stands, untuned) on whole layer-steps of the workload: one layer's cache,
    whole path, with all host threads for about budget_s seconds, then with one thread on a slice of the KV
    heads (heads are independent in every pass) scaled to the layer."""
    import numpy as np
    import oracle
    import ts_synth as S

    bits = S.torch_bf16_to_bits
    q, k, v = bits(x["q"]), bits(x["k"]), bits(x["v"])
    q_tree, k_tree, v_tree = bits(x["q_tree"]), bits(x["k_tree"]), bits(x["v_tree"])

    def whole_path(q, k, v, q_tree, k_tree, v_tree):
        sc = oracle.chunk_scores(q, k, cfg.chunk, cfg.scale)
        idx = oracle.topk_chunks(sc.astype(np.float32), cfg.n_sink, cfg.k)
        oracle.partial_attn(q, k, v, idx, cfg.chunk, cfg.scale)
        oracle.tree_verify(q_tree, k, v, k_tree, v_tree, x["parent"], cfg.scale)

    reps, t0 = 0, time.perf_counter()
    while True:
        whole_path(q, k, v, q_tree, k_tree, v_tree)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= budget_s or reps >= 64:
            break
    all_threads = oracle.num_threads()
    # one thread: a slice of the KV heads whose work is about 1/8 of the all-threads sample
    hs = max(1, min(cfg.n_kv_heads, int(round(cfg.n_kv_heads * min(1.0, 6.0 * reps / (dt * all_threads))))))
    g = cfg.group
    oracle.set_threads(1)
    try:
        t1 = time.perf_counter()
        whole_path(np.ascontiguousarray(q[:hs * g]), np.ascontiguousarray(k[:hs]), np.ascontiguousarray(v[:hs]),
                   np.ascontiguousarray(q_tree[:, :hs * g]), np.ascontiguousarray(k_tree[:, :hs]),
                   np.ascontiguousarray(v_tree[:, :hs]))
        dt1 = time.perf_counter() - t1
    finally:
        oracle.set_threads(all_threads)
    return {"value": round(dt * 1e6 / reps, 1), "unit": "us/layer-step", "cores": all_threads,
            "kind": "oracle", "seconds_measured": round(dt + dt1, 2),
            "sample": "fp64 oracle (OpenMP over heads/rows), whole path (scores, top-k, partial attention, tree-verify) "
                      "on one layer's cache of the workload, all %d KV heads, %d repetitions" % (cfg.n_kv_heads, reps),
            "single_thread": {"value": round(dt1 * 1e6 * cfg.n_kv_heads / hs, 1), "unit": "us/layer-step", "cores": 1,
                              "sample": "the same path on %d of the %d KV heads of that layer, one thread, once; scaled by %d/%d"
                                        % (hs, cfg.n_kv_heads, cfg.n_kv_heads, hs)}}


def timed(fn, reps):
    """ms per call of fn over reps calls, HIP events on the current stream (the one the library launches on)."""
    import torch
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


class Workload:
    """One workload's layer caches and buffers on the device, and the calls of the path over them."""

    def __init__(self, cfg, dev, n_layers=0, n_tree=0, layers=None):
        import torch
        import paper_2502_18890_amd as ts
        import ts_synth as S
        self.ts, self.cfg, self.dev = ts, cfg, dev
        n_layers = n_layers or cfg.n_layers
        layer_bytes = cfg.n_kv_heads * cfg.n_tokens * cfg.head_dim * 2 * 2
        while n_layers * layer_bytes < (2 << 30):   # small configs: a rotating set well beyond the on-die caches
            n_layers += cfg.n_layers
        self.n_layers = n_layers
        self.t = t = n_tree or cfg.n_tree
        hq, hkv, n = cfg.n_q_heads, cfg.n_kv_heads, cfg.n_tokens
        if layers is not None:     # the caches of another workload object (same shape), with this tree's own q/k/v
            gen = torch.Generator(device=dev)
            gen.manual_seed(cfg.seed * 7919 + t)
            rnd = lambda *s: torch.randn(*s, generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
            self.layers = []
            for x in layers[:n_layers]:
                y = dict(x)
                y["q_tree"], y["k_tree"], y["v_tree"] = rnd(t, hq, cfg.head_dim), rnd(t, hkv, cfg.head_dim), rnd(t, hkv, cfg.head_dim)
                y["q_tree"][0] = x["q"]
                y["parent"] = paper_width_tree() if t == 100 else S.tree_parents(cfg, 0, t, "random")
                self.layers.append(y)
        else:
            self.layers = [S.make_layer_torch(cfg, l, dev, n_tree=t, tree_kind=None if t == cfg.n_tree else "random")
                           for l in range(n_layers)]
            if t == 100:
                for x in self.layers:
                    x["parent"] = paper_width_tree()
        u8 = lambda nbytes: torch.empty(nbytes, dtype=torch.uint8, device=dev)
        self.ws_v = u8(ts.workspace_bytes(ts.OP_TREE_VERIFY, hq, hkv, n, t))
        self.ws_vs = u8(ts.workspace_bytes(ts.OP_TREE_VERIFY_SCORED, hq, hkv, n, t))
        self.ws_p = u8(ts.workspace_bytes(ts.OP_PARTIAL_ATTN, hq, hkv, n, 0, cfg.n_sel, cfg.chunk))
        self.scores = torch.empty(hkv, cfg.n_chunks, dtype=torch.float32, device=dev)
        self.idx = torch.empty(hkv, cfg.n_sel, dtype=torch.int32, device=dev)
        self.out_p = torch.empty(hq, cfg.head_dim, dtype=torch.float32, device=dev)
        self.out_v = torch.empty(t, hq, cfg.head_dim, dtype=torch.float32, device=dev)
        self.alg_bytes = (hkv * n * cfg.head_dim * 2 * 2 + t * hkv * cfg.head_dim * 2 * 2 + t * hq * cfg.head_dim * 2
                          + t * hq * cfg.head_dim * 4)
        # algorithmic flops = QK^T and PV once each, 4*g*T*d flops per cached or tree key and KV head (the second,
        # low-order PV product that keeps the weights' precision is an implementation cost and is not counted)
        self.alg_flops = 4.0 * cfg.group * t * cfg.head_dim * (n + t) * hkv
        torch.cuda.synchronize()

    # the calls, one layer each
    def do_scores(self, x):
        self.ts.chunk_scores(x["q"], x["k"], self.cfg.chunk, self.cfg.scale, out=self.scores)

    def do_topk(self, x):
        self.ts.topk_chunks(self.scores, self.cfg.n_sink, self.cfg.k, out=self.idx)

    def do_partial(self, x):
        self.ts.partial_kv_attn(x["q"], x["k"], x["v"], self.idx, self.cfg.chunk, self.cfg.scale, out=self.out_p, workspace=self.ws_p)

    def do_verify(self, x):
        self.ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], self.cfg.scale,
                                 out=self.out_v, workspace=self.ws_v)

    def do_verify_scored(self, x):
        # the verification pass also leaves the chunk scores for the query of tree node 0 (= x["q"] in these inputs)
        self.ts.tree_verify_attn(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], self.cfg.scale,
                                 out=self.out_v, workspace=self.ws_vs, score_chunk=self.cfg.chunk, scores=self.scores)

    def do_split_kernel(self, x, scored):
        self.ts.bench_verify_split_kernel(x["q_tree"], x["k"], x["v"], x["k_tree"], x["v_tree"], x["parent"], self.cfg.scale,
                                          self.ws_vs if scored else self.ws_v, with_tile_sums=scored)

    def step_four_pass(self):
        for x in self.layers:
            self.do_scores(x)
            self.do_topk(x)
            self.do_partial(x)
            self.do_verify(x)

    def step_scored(self):
        # the order of Alg. 1: verification over the full cache (whose query-key products give the scores),
        # rebuild of the partial cache's chunk list, drafting pass over it
        for x in self.layers:
            self.do_verify_scored(x)
            self.do_topk(x)
            self.do_partial(x)

    def sweep(self, fn):
        return lambda: [fn(x) for x in self.layers]

    def split_kernel_us(self, scored, loops):
        """Average duration of the verification pass's split kernel alone over at least `loops` sweeps of the layers and at
        least 20 ms (HIP events on the launch stream).  Untimed sweeps come first until the chip has run this kernel for
        40 ms: the power limit sets the clock of the wide passes, and for the first milliseconds after lighter work the
        clock is still settling (a 128-row pass was seen at 84 us there against 67 us sustained)."""
        import time
        fn = self.sweep(lambda x: self.do_split_kernel(x, scored))
        t0 = time.perf_counter()
        sweep_ms = timed(fn, 1)
        while (time.perf_counter() - t0) * 1e3 < 40.0:
            timed(fn, 1)
        reps = max(1, loops, int(20.0 / max(sweep_ms, 1e-3)) + 1)
        return timed(fn, reps) * 1e3 / self.n_layers

    def kernel_rooflines(self, kern_us):
        gbs = self.alg_bytes / (kern_us * 1e-6) / 1e9
        tf = self.alg_flops / (kern_us * 1e-6) / 1e12
        return gbs, tf

    def graph_of(self, step):
        import torch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            step()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        return graph

    def brief(self, steps, warmup, kernel_loops, with_graph=False):
        """Step (both ways), verification kernel alone and its roofline fractions."""
        for _ in range(max(1, warmup)):
            self.step_scored()
        self.step_four_pass()
        us = timed(self.step_scored, steps) * 1e3 / self.n_layers
        us4 = timed(self.step_four_pass, max(2, steps // 2)) * 1e3 / self.n_layers
        kern_us = self.split_kernel_us(True, kernel_loops)
        kern_plain_us = self.split_kernel_us(False, kernel_loops)
        gbs, tf = self.kernel_rooflines(kern_us)
        cfg = self.cfg
        rows = cfg.group * self.t
        res = {"name": "%s: %d q heads / %d kv heads, N=%d, tree %d nodes (%d query rows per KV head), %d layer caches"
                       % (cfg.name, cfg.n_q_heads, cfg.n_kv_heads, cfg.n_tokens, self.t, rows, self.n_layers),
               "value": round(us, 3), "value_no_reading": round(us4, 3), "unit": "us/layer-step",
               "verify_kernel_us": round(kern_us, 3), "verify_kernel_plain_us": round(kern_plain_us, 3),
               "verify_kernel": "verify_dma_kernel" if rows <= 32 else "verify_wide_kernel",
               "hbm_gbs": round(gbs, 1), "hbm_frac": round(gbs / HBM_PEAK_GBS, 4),
               "mfma_tflops": round(tf, 2), "mfma_frac": round(tf / MFMA_PEAK_TFLOPS, 4),
               "algorithmic_bytes_per_launch": self.alg_bytes, "algorithmic_flops_per_launch": self.alg_flops}
        if with_graph:
            graph = self.graph_of(self.step_scored)
            res["value_graph_replay"] = round(timed(graph.replay, steps) * 1e3 / self.n_layers, 3)
        return res


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
    ci = HEADLINE if args.config is None else args.config
    cfg = S.CONFIGS[ci]
    if args.splits:
        ts.tune_set("verify_splits", args.splits)
    w = Workload(cfg, dev, args.layers, args.tree)
    layers, n_layers, t = w.layers, w.n_layers, w.t
    if args.zero_cache:
        for x in layers:
            x["k"].zero_()
            x["v"].zero_()
    hq, hkv, n = cfg.n_q_heads, cfg.n_kv_heads, cfg.n_tokens
    scores, idx = w.scores, w.idx

    step = w.step_four_pass if args.four_pass else w.step_scored
    other_step = w.step_scored if args.four_pass else w.step_four_pass

    for _ in range(args.warmup):
        step()
    other_step()
    torch.cuda.synchronize()
    # both ways of getting the scores select the same chunks (same query, same keys; sums in another order)
    x0 = layers[0]
    w.do_scores(x0); w.do_topk(x0)
    idx_a = idx.clone()
    w.do_verify_scored(x0); w.do_topk(x0)
    same_sets = sum(len(set(a.tolist()) & set(b.tolist())) for a, b in zip(idx_a.cpu(), idx.cpu())) / float(idx.numel())
    assert same_sets > 0.98 or args.zero_cache, "scores from the verification pass select other chunks than the scoring pass (%.3f)" % same_sets
    if args.hold > 0:
        t_start, calls = time.time(), 0
        sink0 = torch.zeros(1, dtype=torch.int32, device=dev)
        while time.time() - t_start < args.hold:
            for x in layers:
                if args.hold_what == "verify":
                    w.do_verify(x)
                else:
                    ts.stream_read_probe(x["k"], sink0)
                    ts.stream_read_probe(x["v"], sink0)
            torch.cuda.synchronize()
            calls += len(layers)
        dt = time.time() - t_start
        if args.hold_what == "verify":
            print("bench.py --hold: %s, tree %d%s%s, %d verification passes in %.1f s, %.1f us each"
                  % (cfg.name, t, ", %d splits" % args.splits if args.splits else "", ", cache of zeros" if args.zero_cache else "",
                     calls, dt, dt / calls * 1e6), flush=True)
        else:
            nbytes = 2 * layers[0]["k"].numel() * 2
            print("bench.py --hold: %s, %d plain reads of one layer's K and V (%d bytes) in %.1f s, %.1f us each, %.0f GB/s"
                  % (cfg.name, calls, nbytes, dt, dt / calls * 1e6, nbytes * calls / dt / 1e9), flush=True)
        return
    run_step = step
    if args.graph:   # the calls allocate nothing and never synchronise, so a step can be captured as it is
        run_step = w.graph_of(step).replay
    wall0 = time.perf_counter()
    ms_per_step = timed(run_step, args.steps)
    wall = time.perf_counter() - wall0
    ms_other = timed(other_step, max(2, args.steps // 2))
    # the same step replayed from a HIP graph (no launch gaps between the five kernels of a layer), beside the eager figure
    graph_us = None
    if not args.graph:
        g = w.graph_of(step)
        graph_us = timed(g.replay, args.steps) * 1e3 / n_layers
        del g

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
             for name, fn in (("scores", w.do_scores), ("topk", w.do_topk), ("partial", w.do_partial), ("verify", w.do_verify),
                              ("verify_scored", w.do_verify_scored))}
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
    w.do_topk(layers[0])
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

    # the dominant kernel alone (split kernel of the verification pass, as the timed step runs it), for the roofline
    kern_us = w.split_kernel_us(not args.four_pass, args.kernel_loops)
    # what plain reading of the same cache buffers sustains (nothing but loads): the practical ceiling
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    probe_bytes = 0

    def do_probe(x):
        ts.stream_read_probe(x["k"], sink)
        ts.stream_read_probe(x["v"], sink)
    if all(x["k"].is_contiguous() and x["v"].is_contiguous() for x in layers):
        probe_bytes = 2 * layers[0]["k"].numel() * 2
        timed(w.sweep(do_probe), 1)
        probe_us = timed(w.sweep(do_probe), max(1, args.kernel_loops)) * 1e3 / n_layers
    alg_bytes, alg_flops = w.alg_bytes, w.alg_flops
    achieved, achieved_tf = w.kernel_rooflines(kern_us)
    kernel_name = "verify_dma_kernel (16x16x32 MFMA)" if cfg.group * t <= 32 else "verify_wide_kernel (32x32x16 MFMA)"

    us_per_layer_step = ms_per_step * 1e3 / n_layers
    us_other = ms_other * 1e3 / n_layers
    # beyond 128 query rows per KV head (beyond 64 with 8 KV heads or more) the verification pass multiplies fp16 weights with fp16 values
    rows = cfg.group * t
    half = rows > 128 or (rows > 64 and hkv >= 8)
    dtype = "bf16 inputs, fp32 accumulate" + (" (weights x values of the verification pass in fp16)" if half else "")
    res = {
        "metric": "us per layer-step: chunk scores + top-k + partial-KV attention + tree-verify attention over the full cache",
        "value": round(us_per_layer_step, 3), "unit": "us/layer-step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": dtype, "data": "synthetic",
        "config": {"workload": "%s: %d q heads / %d kv heads, d=128, N=%d cached tokens, chunk %d, top-k %d+%d chunks, tree %d nodes, %d layer caches, batch 1" % (
            cfg.name, hq, hkv, n, cfg.chunk, cfg.k, cfg.n_sink, t, n_layers), "config_index": ci,
            "layers": n_layers, "n_tokens": n, "launch": "hip graph replay" if args.graph else "eager"},
        "step": ("four passes: ts_chunk_scores, ts_topk_chunks, ts_partial_kv_attn, ts_tree_verify_attn" if args.four_pass else
                 "three passes: ts_tree_verify_attn_scored (verification; its query-key products of tree node 0 also give the "
                 "chunk scores, same values as ts_chunk_scores for that query), ts_topk_chunks, ts_partial_kv_attn"),
        # the step that assumes nothing about which query ranks the cache: the scores are a pass of their own
        "value_graph_replay": round(us_per_layer_step if args.graph else graph_us, 3),
        "value_no_reading": round(us_per_layer_step if args.four_pass else us_other, 3),
        "value_scores_left_to_verification": round(us_other if args.four_pass else us_per_layer_step, 3),
        "reading": "value_scores_left_to_verification holds if the query that ranks the cache is the verification pass's query "
                   "of tree node 0 (Sec. 3.3 names query-key products, not the pass or the query); value_no_reading holds for any query",
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
                     "traffic": measured_traffic(cfg.name, ts.version()) if (n == cfg.n_tokens and t == cfg.n_tree) else None,
                     "algorithmic_bytes_per_launch": alg_bytes, "avg_launch_us": round(kern_us, 3)},
        "stream_read_ceiling": ({"GBps": round(probe_bytes / (probe_us * 1e-6) / 1e9, 1), "bytes_per_layer": probe_bytes,
                                 "us_per_layer": round(probe_us, 3),
                                 "frac_of_peak": round(probe_bytes / (probe_us * 1e-6) / 1e9 / HBM_PEAK_GBS, 4),
                                 "roofline_kernel_frac_of_ceiling": round(achieved / (probe_bytes / (probe_us * 1e-6) / 1e9), 4),
                                 "what": "a kernel of nothing but 128-bit loads over the same K and V buffers, same rotation"}
                                if probe_bytes else None),
        "roofline_mfma": {"bound": "mfma", "achieved": round(achieved_tf, 2), "peak": MFMA_PEAK_TFLOPS,
                          "unit": "TFLOP/s", "frac": round(achieved_tf / MFMA_PEAK_TFLOPS, 4),
                          "algorithmic_flops_per_launch": alg_flops, "flops_per_byte": round(alg_flops / alg_bytes, 1)},
        "library_version": ts.version(),
    }
    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            torch.add(a, 1.0, out=b)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, layers[0])

    if args.config is None and not args.tree and not args.layers and not args.splits and not args.zero_cache:
        # the other workloads in brief: the paper's verification width on the headline caches, then the two large
        # GQA shapes (the first of them also at the paper's verification width); the two small shapes eager and as a graph replay
        steps = max(4, args.steps // 2)
        others = [Workload(cfg, dev, 0, 100, layers=layers).brief(steps, 1, args.kernel_loops)]
        del w, layers, x0
        torch.cuda.empty_cache()
        for cj in (2, 4):
            wj = Workload(S.CONFIGS[cj], dev)
            others.append(wj.brief(steps, 1, args.kernel_loops))
            if cj == 2:   # the paper's verification width on a GQA shape: 400 query rows per KV head, two row tiles
                others.append(Workload(S.CONFIGS[cj], dev, 0, 100, layers=wj.layers).brief(steps, 1, args.kernel_loops))
            del wj
            torch.cuda.empty_cache()
        res["workloads"] = others
        small = []
        for cj in (0, 1):
            wj = Workload(S.CONFIGS[cj], dev)
            small.append(wj.brief(steps, 1, args.kernel_loops, with_graph=True))
            del wj
            torch.cuda.empty_cache()
        res["small_workloads"] = small
    print(json.dumps(res))


if __name__ == "__main__":
    main()
