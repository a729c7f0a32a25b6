"""GPU parity: every entry point of the C ABI against the fp64 oracle, element by element, on
the same seeded inputs (sizes that span several tiles and ragged tails, plus edge cases)."""
import math

import numpy as np
import pytest

import oracle
import ts_synth as S
from gpu_util import assert_close, dev
from helpers import rand_bits

pytestmark = pytest.mark.gpu

D = 128
SCALE = 1.0 / math.sqrt(D)


@pytest.fixture(scope="module")
def ts():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18890_amd as lib
    lib.load_library()
    return lib


def _np(t):
    return t.detach().cpu().numpy()


def _case(seed, hq, hkv, n, t, vscale=1.0, kscale=1.0):
    rng = np.random.default_rng(seed)
    return dict(q=rand_bits(rng, hq, D), q_tree=rand_bits(rng, t, hq, D), k_tree=rand_bits(rng, t, hkv, D, scale=kscale),
                v_tree=rand_bits(rng, t, hkv, D, scale=vscale), k=rand_bits(rng, hkv, max(n, 1), D, scale=kscale)[:, :n],
                v=rand_bits(rng, hkv, max(n, 1), D, scale=vscale)[:, :n], rng=rng)


def _random_parent(rng, t):
    p = np.full(t, -1, dtype=np.int32)
    for i in range(1, t):
        p[i] = rng.integers(-1, i)     # -1 allowed: forests with several roots
    return p


# ------------------------------------------------------------------------------------------
# chunk scores
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("hq,hkv,n,chunk", [(4, 1, 4096, 64), (12, 2, 16384, 64), (32, 8, 1000, 64),
                                            (32, 32, 1567, 64), (40, 8, 777, 64), (6, 1, 300, 16),
                                            (8, 1, 257, 128), (4, 2, 130, 1), (7, 7, 5, 64), (16, 2, 3000, 1000),
                                            (3, 1, 100, 48)])
def test_chunk_scores(ts, hq, hkv, n, chunk):
    c = _case(1, hq, hkv, n, 1)
    got = ts.chunk_scores(dev(c["q"]), dev(c["k"]), chunk, SCALE)
    ref = oracle.chunk_scores(c["q"], c["k"], chunk, SCALE)
    assert_close(_np(got), ref, "chunk_scores")


def test_chunk_scores_token_major_layout(ts):
    """K stored [N, Hkv, d] and passed as a strided [Hkv, N, d] view."""
    rng = np.random.default_rng(2)
    hq, hkv, n = 8, 4, 1234
    q = rand_bits(rng, hq, D)
    k_tm = rand_bits(rng, n, hkv, D)
    got = ts.chunk_scores(dev(q), dev(k_tm).transpose(0, 1), 64, SCALE)
    ref = oracle.chunk_scores(q, k_tm.transpose(1, 0, 2), 64, SCALE)
    assert_close(_np(got), ref, "chunk_scores token-major")


# ------------------------------------------------------------------------------------------
# top-k: bit-exact from the same fp32 score vector
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("hkv,n_chunks,n_sink,k", [(1, 64, 1, 8), (2, 256, 1, 64), (8, 1024, 1, 64), (32, 1563, 1, 64),
                                                   (8, 1600, 1, 128), (3, 1, 1, 0), (3, 1, 0, 1), (2, 2, 0, 2),
                                                   (2, 17, 3, 14), (1, 8192, 2, 512), (4, 100, 0, 100), (2, 33, 33, 0),
                                                   (2, 300, 0, 256), (2, 300, 1, 257), (3, 8193, 0, 4096), (2, 9000, 3, 100),
                                                   (1, 100000, 0, 4096), (2, 70000, 64, 8192), (2, 255, 0, 1), (2, 257, 1, 256),
                                                   (1, 65537, 1, 17), (2, 5000, 0, 5000)])
def test_topk_matches_oracle_bit_exact(ts, hkv, n_chunks, n_sink, k):
    import torch
    rng = np.random.default_rng(3)
    s = rng.standard_normal((hkv, n_chunks)).astype(np.float32)
    s[:, ::5] = np.round(s[:, ::5] * 2) / 2            # many exact ties
    got = ts.topk_chunks(torch.from_numpy(s).cuda(), n_sink, k)
    ref = oracle.topk_chunks(s, n_sink, k)
    np.testing.assert_array_equal(_np(got), ref)


def test_topk_special_values(ts):
    import torch
    s = np.array([[5.0, 1.0, 1.0, -0.0, 0.0, np.nan, 1.0, np.nan, -np.inf, np.inf, -1e-45, 1e-45, 3.4e38, -3.4e38]],
                 dtype=np.float32)
    for n_sink in (0, 1, 2):
        k = s.shape[1] - n_sink
        got = ts.topk_chunks(torch.from_numpy(s).cuda(), n_sink, k)
        np.testing.assert_array_equal(_np(got), oracle.topk_chunks(s, n_sink, k))
    s = np.full((2, 70), 0.25, dtype=np.float32)
    np.testing.assert_array_equal(_np(ts.topk_chunks(torch.from_numpy(s).cuda(), 1, 40)), oracle.topk_chunks(s, 1, 40))
    # all scores equal over more chunks than one index digit covers: the cut is decided by the index alone
    for n, k in ((5000, 100), (5000, 3000), (70000, 2049)):
        s = np.full((2, n), -1.5, dtype=np.float32)
        np.testing.assert_array_equal(_np(ts.topk_chunks(torch.from_numpy(s).cuda(), 2, k)), oracle.topk_chunks(s, 2, k))


def test_scores_then_topk_pipeline(ts):
    """Scores from the GPU feed both selections: indices must agree exactly; and with the planted
    chunks of the tiny config the oracle's own fp64 scores select the same set."""
    cfg = S.CONFIGS[0]
    x = S.make_layer(cfg, 0)
    sc = ts.chunk_scores(dev(x["q"]), dev(x["k"]), cfg.chunk, cfg.scale)
    idx = _np(ts.topk_chunks(sc, cfg.n_sink, cfg.k))
    np.testing.assert_array_equal(idx, oracle.topk_chunks(_np(sc), cfg.n_sink, cfg.k))
    ref_idx = oracle.topk_chunks(oracle.chunk_scores(x["q"], x["k"], cfg.chunk, cfg.scale), cfg.n_sink, cfg.k)
    assert set(idx[0].tolist()) == set(ref_idx[0].tolist())


# ------------------------------------------------------------------------------------------
# partial-KV attention
# ------------------------------------------------------------------------------------------
@pytest.mark.parametrize("ci", [0, 1])
def test_partial_attn_configs(ts, ci):
    cfg = S.CONFIGS[ci]
    x = S.make_layer(cfg, 0)
    sc = oracle.chunk_scores(x["q"], x["k"], cfg.chunk, cfg.scale)
    idx = oracle.topk_chunks(sc, cfg.n_sink, cfg.k)
    import torch
    out, lse = ts.partial_kv_attn(dev(x["q"]), dev(x["k"]), dev(x["v"]), torch.from_numpy(idx).cuda(), cfg.chunk,
                                  cfg.scale, want_lse=True)
    ref, rlse = oracle.partial_attn(x["q"], x["k"], x["v"], idx, cfg.chunk, cfg.scale)
    assert_close(_np(out), ref, "partial out")
    assert_close(_np(lse), rlse, "partial lse")


@pytest.mark.parametrize("hq,hkv,n,chunk,sel", [
    (4, 1, 300, 64, [[4, 0, 2]]),                 # last chunk has 44 tokens
    (8, 8, 65, 64, [[1, 0]] * 8),                 # last chunk has 1 token
    (5, 1, 1, 64, [[0]]),                         # single key
    (6, 1, 17, 16, [[1, 0]]),                     # chunk 16, 1-token tail
    (16, 2, 1000, 128, [[7, 3, 0], [0, 1, 2]]),   # chunk 128, 104-token tail
    (8, 1, 200, 32, [[6, 6, 1]]),                 # a chunk listed twice counts twice
    (2, 2, 4096, 64, [list(range(64))] * 2),      # every chunk: full attention
    (3, 3, 640, 64, [[9, 8, 7, 6, 5, 4, 3, 2, 1, 0]] * 3),
])
def test_partial_attn_edges(ts, hq, hkv, n, chunk, sel):
    import torch
    c = _case(5, hq, hkv, n, 1, vscale=2.0)
    idx = np.asarray(sel, dtype=np.int32)
    out, lse = ts.partial_kv_attn(dev(c["q"]), dev(c["k"]), dev(c["v"]), torch.from_numpy(idx).cuda(), chunk, SCALE,
                                  want_lse=True)
    ref, rlse = oracle.partial_attn(c["q"], c["k"], c["v"], idx, chunk, SCALE)
    assert_close(_np(out), ref, "partial out")
    assert_close(_np(lse), rlse, "partial lse")


# ------------------------------------------------------------------------------------------
# tree verification attention
# ------------------------------------------------------------------------------------------
def _verify_both(ts, c, parent, scale=SCALE, layout="head"):
    n = c["k"].shape[1]
    if n == 0:
        kd = vd = None
    elif layout == "head":
        kd, vd = dev(c["k"]), dev(c["v"])
    else:   # token-major storage, strided view
        kd = dev(np.ascontiguousarray(c["k"].transpose(1, 0, 2))).transpose(0, 1)
        vd = dev(np.ascontiguousarray(c["v"].transpose(1, 0, 2))).transpose(0, 1)
    out, lse = ts.tree_verify_attn(dev(c["q_tree"]), kd, vd, dev(c["k_tree"]), dev(c["v_tree"]), parent, scale,
                                   want_lse=True)
    ref, rlse = oracle.tree_verify(c["q_tree"], c["k"] if n else None, c["v"] if n else None, c["k_tree"],
                                   c["v_tree"], parent, scale)
    return _np(out), _np(lse), ref, rlse


@pytest.mark.parametrize("ci", [0, 1])
def test_verify_configs(ts, ci):
    cfg = S.CONFIGS[ci]
    x = S.make_layer(cfg, 0)
    out, lse, ref, rlse = _verify_both(ts, x, x["parent"], cfg.scale)
    assert_close(out, ref, "verify out")
    assert_close(lse, rlse, "verify lse")


@pytest.mark.parametrize("hq,hkv,n,t", [
    (4, 1, 0, 8), (4, 1, 1, 1), (4, 4, 31, 5), (8, 2, 32, 16), (8, 2, 33, 16), (6, 1, 63, 7), (5, 1, 64, 13),
    (12, 2, 65, 16), (32, 8, 4096 + 17, 32), (32, 32, 1000, 32), (40, 8, 2100, 64), (6, 1, 500, 64),
    (8, 1, 300, 64), (8, 1, 700, 33), (16, 2, 257, 20), (7, 1, 129, 3), (2, 2, 97, 64), (3, 3, 5000, 2),
    (8, 1, 100, 128), (32, 4, 64, 128), (5, 5, 1, 65), (1, 1, 40, 127), (24, 8, 350, 70),
])
def test_verify_shapes(ts, hq, hkv, n, t):
    c = _case(7, hq, hkv, n, t)
    parent = _random_parent(c["rng"], t)
    out, lse, ref, rlse = _verify_both(ts, c, parent)
    assert_close(out, ref, "verify out")
    assert_close(lse, rlse, "verify lse")


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("hq,hkv,n,t,chunk", [
    (4, 4, 1000, 8, 64), (32, 32, 1567, 32, 64), (8, 2, 2500, 16, 32), (32, 8, 4133, 32, 64), (40, 8, 3001, 64, 128),
    (6, 2, 777, 5, 32), (12, 2, 16384, 16, 64), (16, 2, 33, 20, 64), (8, 8, 1, 3, 32), (48, 8, 2300, 100, 96),
    (64, 8, 900, 128, 1024), (5, 1, 6500, 7, 64),
])
def test_verify_scored_leaves_the_chunk_scores_of_the_root_query(ts, variant, hq, hkv, n, t, chunk):
    """The scored call returns the same attention output as the plain one, bit for bit, and the chunk
    scores that the scoring pass gives for the query of tree node 0 -- for every kernel shape (rows of
    node 0 in the 16x16x32 kernel, in the first row block of the 32x32x16 kernel, with key groups)."""
    import torch
    c = _case(33, hq, hkv, n, t)
    parent = _random_parent(c["rng"], t)
    args = (dev(c["q_tree"]), dev(c["k"]), dev(c["v"]), dev(c["k_tree"]), dev(c["v_tree"]), parent, SCALE)
    try:
        ts.tune_set("verify_variant", variant)
        plain = ts.tree_verify_attn(*args)
        out, lse, scores = ts.tree_verify_attn(*args, want_lse=True, score_chunk=chunk)
    finally:
        ts.tune_set("verify_variant", 0)
    assert torch.equal(plain, out)
    ref, rlse = oracle.tree_verify(c["q_tree"], c["k"], c["v"], c["k_tree"], c["v_tree"], parent, SCALE)
    assert_close(_np(out), ref, "scored verify out")
    assert_close(_np(lse), rlse, "scored verify lse")
    assert_close(_np(scores), oracle.chunk_scores(c["q_tree"][0], c["k"], chunk, SCALE), "scores from the verification pass")
    # the same numbers as the scoring pass proper, to rounding order
    direct = ts.chunk_scores(dev(c["q_tree"])[0].contiguous(), dev(c["k"]), chunk, SCALE)
    np.testing.assert_allclose(_np(scores), _np(direct), rtol=0, atol=2e-4)


def test_verify_scored_token_major_layout(ts):
    """K and V stored [N, Hkv, d] and passed as strided views: same scores, same output."""
    c = _case(34, 8, 2, 1500, 12)
    parent = _random_parent(c["rng"], 12)
    kd = dev(np.ascontiguousarray(c["k"].transpose(1, 0, 2))).transpose(0, 1)
    vd = dev(np.ascontiguousarray(c["v"].transpose(1, 0, 2))).transpose(0, 1)
    out, scores = ts.tree_verify_attn(dev(c["q_tree"]), kd, vd, dev(c["k_tree"]), dev(c["v_tree"]), parent, SCALE, score_chunk=64)
    assert_close(_np(out), oracle.tree_verify(c["q_tree"], c["k"], c["v"], c["k_tree"], c["v_tree"], parent, SCALE)[0], "out")
    assert_close(_np(scores), oracle.chunk_scores(c["q_tree"][0], c["k"], 64, SCALE), "scores")


@pytest.mark.parametrize("kind", ["chain", "star", "fixed"])
def test_verify_tree_kinds(ts, kind):
    c = _case(8, 8, 2, 200, 8)
    parent = S.tree_parents(S.CONFIGS[0], 0, 8, kind)
    out, lse, ref, rlse = _verify_both(ts, c, parent)
    assert_close(out, ref, "verify out")
    assert_close(lse, rlse, "verify lse")


def test_verify_token_major_layout(ts):
    c = _case(9, 8, 4, 777, 9)
    parent = _random_parent(c["rng"], 9)
    out, lse, ref, rlse = _verify_both(ts, c, parent, layout="token")
    assert_close(out, ref, "verify out")
    assert_close(lse, rlse, "verify lse")


def test_verify_dominant_key_and_large_values(ts):
    """One key with a logit about +20 above the rest, values 8x larger: the weights are peaked,
    so rounding the probabilities would show directly in the output."""
    c = _case(10, 8, 2, 600, 12, vscale=8.0)
    kf = S.bf16_bits_to_f32(c["k"]).copy()
    qf = S.bf16_bits_to_f32(c["q_tree"])
    for h in range(2):
        kf[h, 123 + h] = qf[3, h * 4] * (20.0 / SCALE / float(qf[3, h * 4] @ qf[3, h * 4]))
    c["k"] = S.f32_to_bf16_bits(kf)
    parent = _random_parent(c["rng"], 12)
    out, lse, ref, rlse = _verify_both(ts, c, parent)
    assert_close(out, ref, "verify out (peaked)")
    assert_close(lse, rlse, "verify lse (peaked)")


@pytest.mark.parametrize("hq,hkv,t", [(32, 8, 64), (40, 8, 64), (16, 4, 64)])
def test_verify_dominant_key_and_large_values_wide(ts, hq, hkv, t):
    """The same with 256 and 320 rows per KV head (the shapes whose second product runs in fp16)
    and with 64: a key that carries nearly all the weight, values 8x larger."""
    g = hq // hkv
    c = _case(40, hq, hkv, 1500, t, vscale=8.0)
    kf = S.bf16_bits_to_f32(c["k"]).copy()
    qf = S.bf16_bits_to_f32(c["q_tree"])
    for h in range(hkv):
        kf[h, 321 + h] = qf[5, h * g] * (20.0 / SCALE / float(qf[5, h * g] @ qf[5, h * g]))
    c["k"] = S.f32_to_bf16_bits(kf)
    parent = _random_parent(c["rng"], t)
    out, lse, ref, rlse = _verify_both(ts, c, parent)
    assert_close(out, ref, "verify out (peaked, wide)")
    assert_close(lse, rlse, "verify lse (peaked, wide)")


@pytest.mark.parametrize("hq,hkv,t", [(32, 8, 64), (40, 8, 64)])
def test_verify_few_keys_precision_wide(ts, hq, hkv, t):
    """Few comparable keys per row at 256 and 320 rows per KV head, values 4x larger."""
    for n in (0, 1, 3):
        c = _case(50 + n, hq, hkv, n, t, vscale=4.0)
        parent = _random_parent(c["rng"], t)
        out, lse, ref, rlse = _verify_both(ts, c, parent)
        assert_close(out, ref, "verify out (few keys, wide, n=%d)" % n)


def test_verify_few_keys_precision(ts):
    """Two or three comparable keys per row (tiny cache): the regime where a bf16 probability
    would cost ~2^-9 of |v|."""
    for n, t in [(1, 2), (2, 1), (3, 4), (0, 3)]:
        c = _case(11 + n, 4, 2, n, t, vscale=4.0)
        parent = np.arange(-1, t - 1, dtype=np.int32)
        out, lse, ref, rlse = _verify_both(ts, c, parent)
        assert_close(out, ref, "verify out (few keys n=%d t=%d)" % (n, t))


def test_verify_split_override_and_determinism(ts):
    """Any number of cache splits gives the same answer to tolerance; the same call twice is
    bit-identical (no atomics anywhere)."""
    c = _case(12, 8, 2, 3000, 16)
    parent = _random_parent(c["rng"], 16)
    base = None
    try:
        for splits in (0, 1, 3, 94):
            ts.tune_set("verify_splits", splits)
            out, lse, ref, rlse = _verify_both(ts, c, parent)
            assert_close(out, ref, "verify out splits=%d" % splits)
            out2, _, _, _ = _verify_both(ts, c, parent)
            np.testing.assert_array_equal(out, out2)
            base = out if base is None else base
    finally:
        ts.tune_set("verify_splits", 0)


@pytest.mark.parametrize("variant", [0, 1, 2, 3])
@pytest.mark.parametrize("hq,hkv,n,t", [(8, 2, 1000, 8), (32, 8, 2085, 32), (12, 2, 999, 16), (40, 8, 700, 64),
                                        (4, 4, 130, 3), (48, 8, 333, 64), (64, 8, 200, 64), (2, 2, 300, 32),
                                        (16, 2, 450, 25), (4, 4, 97, 128), (32, 8, 260, 100), (16, 2, 129, 128), (32, 8, 70, 32),
                                        (40, 8, 31, 64), (20, 4, 1, 60)])
def test_verify_kernel_variants(ts, variant, hq, hkv, n, t):
    """Every kernel shape (the 16x16x32 kernel for few rows, the 32x32x16 kernel in its
    alternative workgroup shapes, row tiles for more than 384 rows) must match the oracle."""
    c = _case(21, hq, hkv, n, t)
    parent = _random_parent(c["rng"], t)
    try:
        ts.tune_set("verify_variant", variant)
        out, lse, ref, rlse = _verify_both(ts, c, parent)
    finally:
        ts.tune_set("verify_variant", 0)
    assert_close(out, ref, "verify out variant=%d" % variant)
    assert_close(lse, rlse, "verify lse variant=%d" % variant)


# every instantiation of the two verification kernels, by its position in the library's list of kernel shapes, with the
# largest number of query rows per KV head it covers (the "verify_kernel" override falls back to the default shape when
# a kernel cannot cover the rows, so each case below really runs the kernel it names)
KERNEL_ROWS = [16, 32, 32, 32, 64, 64, 128, 128, 256, 256, 320, 384, 64, 128, 128, 256, 320, 384, 128, 128, 128, 256]
ROW_SHAPES = {16: [(4, 4, 16), (2, 2, 5)], 32: [(8, 4, 16), (4, 4, 23)], 64: [(8, 2, 16), (12, 4, 17)], 128: [(32, 8, 32), (4, 4, 100), (8, 2, 27)],
              256: [(32, 8, 64), (8, 2, 51)], 320: [(40, 8, 64), (10, 2, 57)], 384: [(48, 8, 64), (6, 1, 61)]}


@pytest.mark.parametrize("kernel_id", range(len(KERNEL_ROWS)))
def test_verify_every_kernel_instantiation(ts, kernel_id):
    """All shapes of the verification kernels, including those no default geometry selects, on a full row count and on a
    ragged one; the cache length leaves a ragged last tile and, for the kernels with key groups, tiles past the end."""
    for hq, hkv, t in ROW_SHAPES[KERNEL_ROWS[kernel_id]]:
        c = _case(40 + kernel_id, hq, hkv, 1229, t)
        parent = _random_parent(c["rng"], t)
        try:
            ts.tune_set("verify_kernel", kernel_id + 1)
            out, lse, ref, rlse = _verify_both(ts, c, parent)
        finally:
            ts.tune_set("verify_kernel", 0)
        assert_close(out, ref, "verify out kernel %d rows %d" % (kernel_id, hq // hkv * t))
        assert_close(lse, rlse, "verify lse kernel %d rows %d" % (kernel_id, hq // hkv * t))


@pytest.mark.parametrize("hq,hkv,n,t", [(32, 8, 2085, 64), (40, 8, 700, 64), (16, 4, 900, 32), (48, 8, 333, 64), (8, 2, 500, 32)])
@pytest.mark.parametrize("kind", ["huge", "tiny"])
@pytest.mark.parametrize("variant", [0, 1, 3])
def test_verify_values_outside_half_range(ts, variant, kind, hq, hkv, n, t):
    """For more than 32 rows per KV head the weights meet V in fp16 when V fits.  Values that do
    not fit -- magnitudes of 65520 and more, or tokens whose values all lie below 2^-14 -- must
    be caught and take the bf16 route: the result still matches the oracle ("tiny": at the bar as it
    stands; "huge": relative to the size of the output, see below)."""
    if kind == "tiny":
        c = _case(31, hq, hkv, n, t, vscale=2.0 ** -30)
    else:
        c = _case(31, hq, hkv, n, t)
        big = S.f32_to_bf16_bits(np.array([131072.0, -1.0e30, 65536.0], dtype=np.float32))
        rng = c["rng"]
        for arr in (c["v"], c["v_tree"]):
            flat = arr.reshape(-1)
            where = rng.choice(flat.size, size=7, replace=False)
            flat[where] = big[rng.integers(0, 3, size=7)]
    parent = _random_parent(c["rng"], t)
    try:
        ts.tune_set("verify_variant", variant)   # 1 and 3 select fp16 shapes for 64 and 128 rows too
        out, lse, ref, rlse = _verify_both(ts, c, parent)
    finally:
        ts.tune_set("verify_variant", 0)
    if kind == "tiny":
        assert_close(out, ref, "verify out, tiny values")          # the bar as it stands (absolute and relative L2)
    else:
        # Stated exception to the absolute bar: with planted values of 1e30 the outputs themselves reach ~1e27,
        # where fp32 has an absolute resolution of ~1e20.  Both sides are divided by the largest reference
        # magnitude before the bar is applied, i.e. max-abs is taken relative to the size of the output.
        size = float(np.max(np.abs(ref)))
        assert size > 1.0e20
        assert_close(out / size, ref / size, "verify out, huge values")
    assert_close(lse, rlse, "verify lse, %s values" % kind)


@pytest.mark.parametrize("hq,hkv,t", [(32, 8, 64), (40, 8, 64), (4, 4, 100)])
def test_verify_small_values_beside_normal_ones_keep_their_bits(ts, hq, hkv, t):
    """Where the second product runs in fp16, values below fp16's normal range (2^-14) sit in subnormals, whose spacing
    of 2^-24 still holds a bf16 value's eight bits down to 2^-17: columns of such values, next to a column of normal
    size (so that no row's output is small as a whole and nothing sends the workgroup to its bf16 pass), must come
    out with their own relative accuracy, not flushed to zero."""
    n = 1500
    c = _case(51, hq, hkv, n, t)
    rng = c["rng"]
    for arr in (c["v"], c["v_tree"]):
        small = (rng.integers(16, 255, size=arr.shape).astype(np.float32) * np.float32(2.0 ** -24))   # 2^-20 .. 2^-16, eight bits each
        small[..., 0] = S.bf16_bits_to_f32(arr[..., 0])                                                # column 0 keeps N(0,1)
        arr[...] = S.f32_to_bf16_bits(small)
    parent = _random_parent(rng, t)
    out, lse, ref, rlse = _verify_both(ts, c, parent)
    assert_close(out, ref, "verify out, small values beside normal ones")
    rel = np.abs(out[..., 1:] - ref[..., 1:]) / np.abs(ref[..., 1:])
    assert float(rel.max()) <= 1e-3, float(rel.max())


@pytest.mark.parametrize("kind", ["chain", "star", "deep-wide"])
def test_verify_wide_trees(ts, kind):
    """Trees of more than 64 nodes (the paper's 40-node tree plus up to 60 retrieved n-gram
    tokens): ancestor masks span both 64-bit words."""
    t = 100
    c = _case(22, 8, 2, 777, t)
    if kind == "chain":
        parent = np.arange(-1, t - 1, dtype=np.int32)
    elif kind == "star":
        parent = np.zeros(t, dtype=np.int32)
        parent[0] = -1
    else:   # 40-node [1,3,3,3] tree, then 20 chains of 3 hanging off the root
        parent = [-1] + [0] * 3 + [1 + i // 3 for i in range(9)] + [4 + i // 3 for i in range(27)]
        for _ in range(20):
            b = len(parent)
            parent += [0, b, b + 1]
        parent = np.asarray(parent, dtype=np.int32)
        assert len(parent) == t
    out, lse, ref, rlse = _verify_both(ts, c, parent)
    assert_close(out, ref, "verify out wide tree " + kind)
    assert_close(lse, rlse, "verify lse wide tree " + kind)
