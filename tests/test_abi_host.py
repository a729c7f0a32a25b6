"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
the header declares, sizes its workspace sanely, and rejects bad arguments before anything
could be launched (no compute call is made here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tokenswift.h")

TS_OK, TS_ERR_NULL, TS_ERR_SHAPE, TS_ERR_UNSUPPORTED = 0, -1, -2, -3
TS_ERR_TREE, TS_ERR_WORKSPACE, TS_ERR_HIP, TS_ERR_ALIGN = -4, -5, -6, -7


@pytest.fixture(scope="module")
def lib():
    from paper_2502_18890_amd import binding
    return binding.load_library()


@pytest.fixture(scope="module")
def binding():
    from paper_2502_18890_amd import binding as b
    return b


def test_library_exports_every_declared_function(lib):
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(ts_[a-z_]+)\s*\(", text)))
    assert names == ["ts_append_accepted", "ts_bench_verify_split_kernel", "ts_chunk_key_sums", "ts_chunk_list_admit", "ts_chunk_scores",
                     "ts_chunk_scores_from_sums", "ts_gather_chunks", "ts_partial_kv_attn", "ts_partial_kv_attn_static", "ts_penalized_probs",
                     "ts_refresh_due", "ts_sample_tokens", "ts_sampling_workspace_bytes", "ts_stream_read_probe", "ts_strerror",
                     "ts_topk_chunks", "ts_tree_verify_attn", "ts_tree_verify_attn_scored", "ts_tune_set", "ts_version", "ts_workspace_bytes"]
    for n in names:
        assert hasattr(lib, n), n
    assert lib.ts_version() >= 100


def test_strerror_covers_all_codes(lib):
    seen = set()
    for code in range(0, -8, -1):
        s = lib.ts_strerror(code).decode()
        assert s and s != "unknown status"
        seen.add(s)
    assert len(seen) == 8
    assert lib.ts_strerror(-99).decode() == "unknown status"


def test_workspace_bytes(binding):
    wb = binding.workspace_bytes
    V, P = binding.OP_TREE_VERIFY, binding.OP_PARTIAL_ATTN
    assert wb(V, 32, 32, 100000, 32) > 0
    assert wb(V, 32, 32, 0, 32) > 0                       # empty cache: tree partial only
    assert wb(V, 32, 32, 100000, 0) == 0                  # no tree
    assert wb(V, 32, 32, 100000, 129) == 0                # tree too large
    assert wb(V, 30, 8, 1000, 8) == 0                     # heads do not divide
    assert wb(V, 72, 8, 1000, 8) == 0                     # group 9 > 8
    assert wb(P, 32, 8, 65536, 0, 65, 64) >= 8 * 17 * 4 * (128 + 2) * 4   # one partial per 16 segments of 16 tokens
    assert wb(P, 32, 8, 65536, 0, 0, 64) == 0             # empty selection
    assert wb(P, 32, 8, 65536, 0, 65, 24) == 0            # chunk not a multiple of 16
    assert wb(99, 32, 8, 65536, 8, 65, 64) == 0
    # the partials must stay a small fraction of the K/V bytes at the benchmark shapes
    for hq, hkv, n, t in [(32, 8, 65536, 32), (32, 32, 100000, 32), (40, 8, 102400, 64)]:
        assert wb(V, hq, hkv, n, t) < 0.3 * hkv * n * 512


def _view(binding, k=0x1000, v=0x2000, n=100, hkv=2, d=128, sh=12800, st=128):
    return binding._KvView(k, v, n, hkv, d, sh, st)


def test_scores_and_topk_reject_bad_arguments(lib, binding):
    q, out = 0x3000, 0x4000
    cs = lambda view, q_=q, hq=4, chunk=64, out_=out: lib.ts_chunk_scores(
        ctypes.byref(view) if view is not None else None, q_, hq, chunk, 1.0, out_, None)
    assert cs(None) == TS_ERR_NULL
    assert cs(_view(binding), q_=None) == TS_ERR_NULL
    assert cs(_view(binding), out_=None) == TS_ERR_NULL
    assert cs(_view(binding, k=None)) == TS_ERR_NULL
    assert cs(_view(binding, d=64)) == TS_ERR_UNSUPPORTED
    assert cs(_view(binding, n=0)) == TS_ERR_SHAPE
    assert cs(_view(binding), hq=3) == TS_ERR_SHAPE
    assert cs(_view(binding), hq=18) == TS_ERR_UNSUPPORTED      # group 9
    assert cs(_view(binding), chunk=0) == TS_ERR_UNSUPPORTED
    assert cs(_view(binding), chunk=2048) == TS_ERR_UNSUPPORTED
    assert cs(_view(binding, k=0x1004)) == TS_ERR_ALIGN
    assert cs(_view(binding, st=132)) == TS_ERR_ALIGN
    assert cs(_view(binding, st=64)) == TS_ERR_SHAPE
    assert cs(_view(binding, st=(1 << 24) + 8)) == TS_ERR_UNSUPPORTED   # token rows too far apart
    tk = lambda n_chunks=10, sink=1, k=3, s=0x1000, o=0x2000: lib.ts_topk_chunks(s, 2, n_chunks, sink, k, o, None)
    assert tk(s=None) == TS_ERR_NULL and tk(o=None) == TS_ERR_NULL
    assert tk(sink=8, k=3) == TS_ERR_SHAPE
    assert tk(sink=0, k=0) == TS_ERR_SHAPE
    assert tk(k=-1) == TS_ERR_SHAPE and tk(sink=-1) == TS_ERR_SHAPE and tk(n_chunks=0) == TS_ERR_SHAPE
    assert tk(n_chunks=(1 << 20) + 1) == TS_ERR_UNSUPPORTED
    assert tk(n_chunks=20000, k=8193) == TS_ERR_UNSUPPORTED


def test_attention_calls_reject_bad_arguments(lib, binding):
    q, idx, out, ws = 0x3000, 0x5000, 0x4000, 0x10000
    big = 1 << 30
    pa = lambda view=None, hq=4, n_sel=3, chunk=64, ws_=ws, wsb=big, q_=q, idx_=idx, out_=out, scale=1.0: lib.ts_partial_kv_attn(
        ctypes.byref(view if view is not None else _view(binding)), q_, hq, idx_, n_sel, chunk, scale, out_, None,
        ws_, wsb, None)
    assert pa(scale=0.0) == TS_ERR_UNSUPPORTED and pa(scale=-1.0) == TS_ERR_UNSUPPORTED
    assert pa(scale=float("inf")) == TS_ERR_UNSUPPORTED and pa(scale=float("nan")) == TS_ERR_UNSUPPORTED
    assert pa(scale=2.5e38) == TS_ERR_UNSUPPORTED          # scale * log2(e) would overflow to infinity
    assert pa(idx_=None) == TS_ERR_NULL and pa(out_=None) == TS_ERR_NULL and pa(q_=None) == TS_ERR_NULL
    assert pa(view=_view(binding, v=None)) == TS_ERR_NULL
    assert pa(n_sel=0) == TS_ERR_SHAPE
    assert pa(n_sel=(1 << 20) + 1) == TS_ERR_UNSUPPORTED          # the segment count would leave 32 bits
    assert pa(chunk=24) == TS_ERR_UNSUPPORTED and pa(chunk=8) == TS_ERR_UNSUPPORTED
    assert pa(ws_=None) == TS_ERR_WORKSPACE and pa(wsb=16) == TS_ERR_WORKSPACE
    assert pa(ws_=ws + 16) == TS_ERR_WORKSPACE                  # not 256-byte aligned
    assert pa(out_=out + 4) == TS_ERR_ALIGN
    # the allocation-free variant: same checks, and its fixed scratch bounds the shape (checked before any device is touched)
    ps = lambda view=None, hq=4, n_sel=3, chunk=64, q_=q, idx_=idx, out_=out, scale=1.0: lib.ts_partial_kv_attn_static(
        ctypes.byref(view if view is not None else _view(binding)), q_, hq, idx_, n_sel, chunk, scale, out_, None, None)
    assert ps(idx_=None) == TS_ERR_NULL and ps(out_=None) == TS_ERR_NULL and ps(n_sel=0) == TS_ERR_SHAPE
    assert ps(chunk=24) == TS_ERR_UNSUPPORTED and ps(scale=0.0) == TS_ERR_UNSUPPORTED
    assert ps(hq=16, n_sel=2100) == TS_ERR_WORKSPACE               # 2 heads x 1050 partials x 8 rows x 520 B > 4 MiB

    def tv(parent, view=None, hq=4, ws_=ws, wsb=big, kt=0x6000, out_=out, scale=1.0):
        par = (ctypes.c_int32 * len(parent))(*parent) if parent is not None else None
        return lib.ts_tree_verify_attn(ctypes.byref(view if view is not None else _view(binding)), q, hq, kt, 0x7000,
                                       par, len(parent) if parent is not None else 4, scale, out_, None, ws_, wsb, None)
    assert tv([-1, 0], scale=0.0) == TS_ERR_UNSUPPORTED and tv([-1, 0], scale=-0.5) == TS_ERR_UNSUPPORTED
    assert tv([-1, 0], scale=float("nan")) == TS_ERR_UNSUPPORTED and tv([-1, 0], scale=2.5e38) == TS_ERR_UNSUPPORTED
    assert tv([-1, 0], view=_view(binding, n=1 << 31)) == TS_ERR_UNSUPPORTED
    assert tv(None) == TS_ERR_NULL
    assert tv([-1, 0], kt=None) == TS_ERR_NULL
    assert tv([0, 0]) == TS_ERR_TREE            # a node cannot be its own parent
    assert tv([-1, 1]) == TS_ERR_TREE           # parent must come earlier
    assert tv([-1, 0, 3]) == TS_ERR_TREE
    assert tv([-2, 0]) == TS_ERR_TREE
    assert tv([]) == TS_ERR_SHAPE
    assert tv([-1] * 129) == TS_ERR_UNSUPPORTED
    assert tv([-1, 0], hq=3) == TS_ERR_SHAPE
    assert tv([-1, 0], ws_=None) == TS_ERR_WORKSPACE and tv([-1, 0], wsb=100) == TS_ERR_WORKSPACE
    assert tv([-1, 0], view=_view(binding, d=96)) == TS_ERR_UNSUPPORTED

    def tvs(parent, chunk=64, scores=0x8000, view=None, wsb=big):
        par = (ctypes.c_int32 * len(parent))(*parent)
        return lib.ts_tree_verify_attn_scored(ctypes.byref(view if view is not None else _view(binding)), q, 4, 0x6000, 0x7000,
                                              par, len(parent), 1.0, chunk, scores, out, None, ws, wsb, None)
    assert tvs([-1, 0], scores=None) == TS_ERR_NULL
    assert tvs([-1, 0], chunk=16) == TS_ERR_UNSUPPORTED and tvs([-1, 0], chunk=48) == TS_ERR_UNSUPPORTED   # whole 32-key tiles only
    assert tvs([-1, 0], chunk=2048) == TS_ERR_UNSUPPORTED
    assert tvs([-1, 0], view=_view(binding, n=0, k=None, v=None)) == TS_ERR_SHAPE      # nothing to score
    assert tvs([0, 0]) == TS_ERR_TREE
    # the scored call needs room for one sum per 32-key tile on top of the plain call's workspace
    need_plain = binding.workspace_bytes(binding.OP_TREE_VERIFY, 4, 2, 100, 2)
    need_scored = binding.workspace_bytes(binding.OP_TREE_VERIFY_SCORED, 4, 2, 100, 2)
    assert need_scored >= need_plain + 2 * 4 * 4
    assert tvs([-1, 0], wsb=need_plain) == TS_ERR_WORKSPACE


def test_bench_split_kernel_entry_rejects_bad_arguments(lib, binding):
    ws, big = 0x10000, 1 << 30
    def sk(parent, view=None, hq=4, sums=0, ws_=ws, wsb=big, q_=0x3000):
        par = (ctypes.c_int32 * len(parent))(*parent)
        return lib.ts_bench_verify_split_kernel(ctypes.byref(view if view is not None else _view(binding)), q_, hq, 0x6000, 0x7000,
                                                par, len(parent), 1.0, sums, ws_, wsb, None)
    assert sk([-1, 0], q_=None) == TS_ERR_NULL and sk([0, 0]) == TS_ERR_TREE and sk([-1, 0], hq=3) == TS_ERR_SHAPE
    assert sk([-1, 0], ws_=None) == TS_ERR_WORKSPACE and sk([-1, 0], wsb=64) == TS_ERR_WORKSPACE
    assert sk([-1, 0], sums=1, view=_view(binding, n=0, k=None, v=None)) == TS_ERR_SHAPE
    need_plain = binding.workspace_bytes(binding.OP_TREE_VERIFY, 4, 2, 100, 2)
    assert sk([-1, 0], sums=1, wsb=need_plain) == TS_ERR_WORKSPACE        # the variant with tile sums needs the larger workspace


def test_tune_set(lib):
    assert lib.ts_tune_set(b"verify_splits", 7) == TS_OK
    assert lib.ts_tune_set(b"verify_splits", 0) == TS_OK
    assert lib.ts_tune_set(b"no_such_knob", 1) == TS_ERR_UNSUPPORTED
    assert lib.ts_tune_set(b"verify_splits", -1) == TS_ERR_UNSUPPORTED
    assert lib.ts_tune_set(None, 1) == TS_ERR_UNSUPPORTED
    assert lib.ts_tune_set(b"verify_stage", 1) == TS_ERR_UNSUPPORTED      # no knob may leave a product call without its output
    assert lib.ts_tune_set(b"verify_variant", 4) == TS_ERR_UNSUPPORTED and lib.ts_tune_set(b"verify_variant", 0) == TS_OK
    assert lib.ts_tune_set(b"verify_kernel", 1000) == TS_ERR_UNSUPPORTED and lib.ts_tune_set(b"verify_kernel", 0) == TS_OK


def test_stream_read_probe_rejects_bad_arguments(lib):
    p = ctypes.c_void_p(4096)
    assert lib.ts_stream_read_probe(None, 1024, p, None) == TS_ERR_NULL
    assert lib.ts_stream_read_probe(p, 1024, None, None) == TS_ERR_NULL
    assert lib.ts_stream_read_probe(p, 0, p, None) == TS_ERR_SHAPE
    assert lib.ts_stream_read_probe(p, 1000, p, None) == TS_ERR_SHAPE              # not a multiple of 16
    assert lib.ts_stream_read_probe(ctypes.c_void_p(4100), 1024, p, None) == TS_ERR_SHAPE   # misaligned
    assert lib.ts_stream_read_probe(p, 1 << 60, p, None) == TS_ERR_UNSUPPORTED


def test_cache_maintenance_calls_reject_bad_arguments(lib, binding):
    """Host-side validation only: every call below must return before anything is enqueued."""
    kt, vt = 0x6000, 0x7000

    def ap(view=None, acc=(0, 1), n_tree=4, kt_=kt, vt_=vt):
        a = (ctypes.c_int32 * max(len(acc), 1))(*acc) if acc is not None else None
        return lib.ts_append_accepted(ctypes.byref(view if view is not None else _view(binding)), kt_, vt_, n_tree, a,
                                      len(acc) if acc is not None else 1, None)
    assert ap(acc=None) == TS_ERR_NULL and ap(kt_=None) == TS_ERR_NULL
    assert ap(view=_view(binding, v=None)) == TS_ERR_NULL
    assert ap(acc=(0, 4)) == TS_ERR_TREE and ap(acc=(-1,)) == TS_ERR_TREE
    assert ap(acc=()) == TS_ERR_SHAPE and ap(n_tree=0) == TS_ERR_SHAPE
    assert ap(acc=tuple([0] * 129), n_tree=4) == TS_ERR_UNSUPPORTED
    assert ap(view=_view(binding, d=64)) == TS_ERR_UNSUPPORTED
    assert ap(view=_view(binding, st=132)) == TS_ERR_ALIGN

    rd = lib.ts_refresh_due
    assert rd(100, 50, 64, 16) == 1 and rd(98, 50, 64, 16) == 0 and rd(99, 50, 64, 16) == 1 and rd(50, 50, 64, 16) == 0
    assert rd(-1, 0, 64, 16) == TS_ERR_SHAPE and rd(10, 11, 64, 16) == TS_ERR_SHAPE and rd(10, 5, 8, 16) == TS_ERR_SHAPE

    ad = lambda idx=0x5000, hkv=2, n_sel=9, sink=1, base=40, first=40, n_new=2: lib.ts_chunk_list_admit(
        idx, hkv, n_sel, sink, base, first, n_new, None)
    assert ad(idx=None) == TS_ERR_NULL
    assert ad(n_new=9) == TS_ERR_SHAPE and ad(n_new=-1) == TS_ERR_SHAPE and ad(base=-3, first=-3) == TS_ERR_SHAPE
    assert ad(first=39) == TS_ERR_SHAPE                              # a chunk from before the rebuild
    assert ad(first=47, n_new=2) == TS_ERR_SHAPE                     # would reach the sink: rebuild instead
    assert ad(sink=10) == TS_ERR_SHAPE and ad(n_new=0) == 0 and ad(first=48, n_new=0) == 0   # nothing to do: no launch

    ga = lambda view=None, idx=0x5000, n_sel=3, chunk=64, ko=0x8000, vo=0x9000: lib.ts_gather_chunks(
        ctypes.byref(view if view is not None else _view(binding)), idx, n_sel, chunk, ko, vo, None)
    assert ga(idx=None) == TS_ERR_NULL and ga(ko=None) == TS_ERR_NULL and ga(vo=None) == TS_ERR_NULL
    assert ga(n_sel=0) == TS_ERR_SHAPE and ga(chunk=24) == TS_ERR_UNSUPPORTED and ga(ko=0x8004) == TS_ERR_ALIGN
    assert ga(view=_view(binding, v=None)) == TS_ERR_NULL

    ks = lambda view=None, chunk=64, cb=0, ce=2, out=0xa000, sh=2 * 128: lib.ts_chunk_key_sums(
        ctypes.byref(view if view is not None else _view(binding)), chunk, cb, ce, out, sh, None)
    assert ks(out=None) == TS_ERR_NULL
    assert ks(ce=3) == TS_ERR_SHAPE and ks(cb=-1) == TS_ERR_SHAPE and ks(cb=2, ce=1) == TS_ERR_SHAPE   # 100 tokens: 2 chunks
    assert ks(chunk=0) == TS_ERR_UNSUPPORTED and ks(sh=128) == TS_ERR_SHAPE and ks(sh=2 * 128 + 2) == TS_ERR_ALIGN
    assert ks(cb=1, ce=1) == 0                                         # empty range: no launch

    sf = lambda ksum=0xa000, sh=2 * 128, hkv=2, n=100, q=0x3000, hq=4, chunk=64, out=0xb000: lib.ts_chunk_scores_from_sums(
        ksum, sh, hkv, n, q, hq, chunk, 1.0, out, None)
    assert sf(ksum=None) == TS_ERR_NULL and sf(q=None) == TS_ERR_NULL and sf(out=None) == TS_ERR_NULL
    assert sf(hq=3) == TS_ERR_SHAPE and sf(hq=18) == TS_ERR_UNSUPPORTED and sf(n=0) == TS_ERR_SHAPE
    assert sf(chunk=2000) == TS_ERR_UNSUPPORTED and sf(sh=128) == TS_ERR_SHAPE


def test_sampling_calls_reject_bad_arguments(lib):
    wsb = lib.ts_sampling_workspace_bytes
    assert wsb(100, 128256) >= 100 * 32 * 8
    assert wsb(0, 1000) == 0 and wsb(4, 0) == 0 and wsb(4, (1 << 24) + 1) == 0
    big = 1 << 30
    pp = lambda lg=0x1000, r=4, v=1000, win=0x3000, nw=8, t=1.0, th=1.2, out=0x2000, ws=0x10000, wb=big: lib.ts_penalized_probs(
        lg, r, v, win, nw, t, th, out, ws, wb, None)
    assert pp(lg=None) == TS_ERR_NULL and pp(out=None) == TS_ERR_NULL and pp(win=None) == TS_ERR_NULL
    assert pp(r=0) == TS_ERR_SHAPE and pp(v=0) == TS_ERR_SHAPE and pp(nw=-1) == TS_ERR_SHAPE
    assert pp(t=0.0) == TS_ERR_UNSUPPORTED and pp(t=float("nan")) == TS_ERR_UNSUPPORTED and pp(th=0.9) == TS_ERR_UNSUPPORTED
    assert pp(v=(1 << 24) + 1) == TS_ERR_UNSUPPORTED
    assert pp(lg=0x1004) == TS_ERR_ALIGN
    assert pp(ws=None) == TS_ERR_WORKSPACE and pp(wb=16) == TS_ERR_WORKSPACE and pp(ws=0x10010) == TS_ERR_WORKSPACE
    st = lambda pr=0x1000, r=4, v=1000, m=1, par=0.1, u=0x3000, tok=0x4000, par2=0.0: lib.ts_sample_tokens(pr, r, v, m, par, par2, u, tok, None, None, None)
    assert st(pr=None) == TS_ERR_NULL and st(u=None) == TS_ERR_NULL and st(tok=None) == TS_ERR_NULL
    assert st(r=0) == TS_ERR_SHAPE and st(v=0) == TS_ERR_SHAPE
    assert st(m=4) == TS_ERR_UNSUPPORTED and st(m=-1) == TS_ERR_UNSUPPORTED
    assert st(m=3, par=0.01, par2=0.0) == TS_ERR_UNSUPPORTED and st(m=3, par=0.0, par2=0.5) == TS_ERR_UNSUPPORTED
    assert st(par=0.0) == TS_ERR_UNSUPPORTED and st(par=1.5) == TS_ERR_UNSUPPORTED and st(m=2, par=float("nan")) == TS_ERR_UNSUPPORTED
