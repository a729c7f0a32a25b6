"""GPU parity of the cache-maintenance calls (through the C ABI) against the numpy oracle:
byte-exact for everything that moves rows or indices, the floating-point bar for the key sums
and the scores computed from them."""
import math

import numpy as np
import pytest

import oracle
import ts_synth as S
from oracle import cache_ops as C
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


def _bits(t):
    return S.torch_bf16_to_bits(t)


@pytest.mark.parametrize("hkv,cap,n,t,acc", [(2, 64, 17, 8, [0, 2, 5]), (8, 300, 0, 4, [3]), (1, 130, 2, 128, list(range(0, 128, 1))),
                                             (32, 40, 31, 9, [0, 1, 4, 8])])
def test_append_accepted_is_byte_exact(ts, hkv, cap, n, t, acc):
    rng = np.random.default_rng(31)
    k, v = rand_bits(rng, hkv, cap, D), rand_bits(rng, hkv, cap, D)
    kt, vt = rand_bits(rng, t, hkv, D), rand_bits(rng, t, hkv, D)
    kd, vd = dev(k), dev(v)
    new_n = ts.append_accepted(kd, vd, n, dev(kt), dev(vt), acc)
    assert new_n == n + len(acc)
    rk, rv = C.append_accepted(k, v, n, kt, vt, acc)
    np.testing.assert_array_equal(_bits(kd), rk)
    np.testing.assert_array_equal(_bits(vd), rv)


def test_append_accepted_token_major_cache(ts):
    """Cache stored [cap, Hkv, d], passed as a strided [Hkv, cap, d] view."""
    rng = np.random.default_rng(32)
    hkv, cap, n, t = 4, 50, 20, 6
    k_tm, v_tm = rand_bits(rng, cap, hkv, D), rand_bits(rng, cap, hkv, D)
    kt, vt = rand_bits(rng, t, hkv, D), rand_bits(rng, t, hkv, D)
    kd, vd = dev(k_tm), dev(v_tm)
    ts.append_accepted(kd.transpose(0, 1), vd.transpose(0, 1), n, dev(kt), dev(vt), [1, 3])
    rk, rv = C.append_accepted(k_tm.transpose(1, 0, 2), v_tm.transpose(1, 0, 2), n, kt, vt, [1, 3])
    np.testing.assert_array_equal(_bits(kd).transpose(1, 0, 2), rk)
    np.testing.assert_array_equal(_bits(vd).transpose(1, 0, 2), rv)


def test_then_verification_sees_the_appended_tokens(ts):
    """After the append the accepted tokens are ordinary cache entries: verifying a one-node tree
    over the grown cache equals the oracle over the grown cache."""
    rng = np.random.default_rng(33)
    hq, hkv, cap, n, t = 8, 2, 700, 650, 12
    k, v = rand_bits(rng, hkv, cap, D), rand_bits(rng, hkv, cap, D)
    kt, vt, qt = rand_bits(rng, t, hkv, D), rand_bits(rng, t, hkv, D), rand_bits(rng, t, hq, D)
    kd, vd = dev(k), dev(v)
    acc = [0, 1, 5, 9]
    new_n = ts.append_accepted(kd, vd, n, dev(kt), dev(vt), acc)
    out = ts.tree_verify_attn(dev(qt[:1]), kd[:, :new_n], vd[:, :new_n], dev(kt[:1]), dev(vt[:1]), [-1], SCALE)
    rk, rv = C.append_accepted(k, v, n, kt, vt, acc)
    ref, _ = oracle.tree_verify(qt[:1], rk[:, :new_n], rv[:, :new_n], kt[:1], vt[:1], np.array([-1], np.int32), SCALE)
    assert_close(out.cpu().numpy(), ref, "verify after append")


@pytest.mark.parametrize("hkv,n_sel,n_sink,base,first,n_new", [(2, 9, 1, 40, 40, 2), (32, 65, 1, 1562, 1563, 3), (3, 5, 0, 7, 7, 5),
                                                               (4, 130, 2, 10, 10, 128), (4, 600, 1, 900, 950, 40), (1, 4, 1, 5, 6, 0)])
def test_chunk_list_admit_is_exact(ts, hkv, n_sel, n_sink, base, first, n_new):
    """Lists without duplicates (as ts_topk_chunks writes them), some of which already hold one or two of
    the chunks being admitted, at a non-sink position or among the sink entries."""
    import torch
    rng = np.random.default_rng(34)
    idx = np.stack([rng.permutation(np.arange(0, first + n_new + 50))[:n_sel] for _ in range(hkv)]).astype(np.int32)
    for h in range(hkv):
        assert len(set(idx[h].tolist())) == n_sel
    got = ts.chunk_list_admit(torch.from_numpy(idx).cuda(), n_sink, base, first, n_new)
    ref = C.chunk_list_admit(idx, n_sink, base, first, n_new)
    np.testing.assert_array_equal(got.cpu().numpy(), ref)
    for h in range(hkv):
        assert len(set(ref[h].tolist())) == n_sel
    # a second, overlapping call (later tokens of the same chunks) changes nothing
    again = ts.chunk_list_admit(got.clone(), n_sink, base, first, n_new)
    np.testing.assert_array_equal(again.cpu().numpy(), ref)


def test_chunk_list_admit_already_listed_cases(ts):
    import torch
    idx = np.array([[0, 7, 12, 9, 5], [0, 2, 8, 4, 12], [12, 3, 8, 4, 6], [0, 13, 12, 4, 6]], dtype=np.int32)
    for n_new in (1, 2):
        got = ts.chunk_list_admit(torch.from_numpy(idx).cuda(), 1, 12, 12, n_new).cpu().numpy()
        np.testing.assert_array_equal(got, C.chunk_list_admit(idx, 1, 12, 12, n_new))


@pytest.mark.parametrize("hkv,n,chunk,n_sel", [(2, 300, 32, 3), (8, 4096, 64, 9), (1, 17, 16, 2), (4, 1000, 128, 5)])
def test_gather_chunks_is_byte_exact(ts, hkv, n, chunk, n_sel):
    import torch
    rng = np.random.default_rng(35)
    k, v = rand_bits(rng, hkv, n, D), rand_bits(rng, hkv, n, D)
    n_chunks = (n + chunk - 1) // chunk
    idx = np.stack([rng.permutation(n_chunks)[:n_sel] for _ in range(hkv)]).astype(np.int32)
    idx[0, -1] = n_chunks - 1                                   # always include the (short) last chunk once
    kg, vg = ts.gather_chunks(dev(k), dev(v), torch.from_numpy(idx).cuda(), chunk)
    rk, rv = C.gather_chunks(k, v, idx, chunk)
    np.testing.assert_array_equal(_bits(kg), rk)
    np.testing.assert_array_equal(_bits(vg), rv)


@pytest.mark.parametrize("hq,hkv,n,chunk", [(4, 1, 4096, 64), (12, 2, 16384, 64), (32, 32, 1567, 64), (40, 8, 777, 64),
                                            (6, 1, 300, 16), (8, 1, 257, 128), (4, 2, 130, 1), (16, 2, 3000, 1000), (3, 1, 100, 48)])
def test_key_sums_and_scores_from_sums(ts, hq, hkv, n, chunk):
    rng = np.random.default_rng(36)
    q, k = rand_bits(rng, hq, D), rand_bits(rng, hkv, n, D)
    kd = dev(k)
    ks = ts.chunk_key_sums(kd, chunk)
    assert_close(ks.cpu().numpy(), C.chunk_key_sums(k, chunk), "key sums")
    sc = ts.chunk_scores_from_sums(ks, n, dev(q), chunk, SCALE)
    ref = oracle.chunk_scores(q, k, chunk, SCALE)               # the definition of the score itself
    assert_close(sc.cpu().numpy(), ref, "scores from sums")
    # and the two GPU routes agree with each other well inside the bar
    direct = ts.chunk_scores(dev(q), kd, chunk, SCALE)
    assert_close(sc.cpu().numpy(), direct.cpu().numpy().astype(np.float64), "sums vs direct", max_abs=2e-5, rel_l2=1e-5)


def test_key_sums_incremental_refresh(ts):
    """Append tokens, refresh only the chunks that changed: equals a full recomputation."""
    rng = np.random.default_rng(37)
    hkv, cap, n0, chunk = 4, 1000, 830, 64
    k = rand_bits(rng, hkv, cap, D)
    kd = dev(k)
    n_cap_chunks = (cap + chunk - 1) // chunk
    import torch
    ks = torch.zeros(hkv, n_cap_chunks, D, dtype=torch.float32, device="cuda")
    ts.chunk_key_sums(kd[:, :n0], chunk, out=ks)
    n1 = n0 + 77                                                # tokens n0 .. n1-1 arrive (already in the buffer)
    ts.chunk_key_sums(kd[:, :n1], chunk, out=ks, chunk_begin=n0 // chunk, chunk_end=(n1 + chunk - 1) // chunk)
    ref = C.chunk_key_sums(k[:, :n1], chunk)
    assert_close(ks.cpu().numpy()[:, :ref.shape[1]], ref, "refreshed sums")
    assert not ks.cpu().numpy()[:, ref.shape[1]:].any()


def test_key_sums_token_major_layout(ts):
    rng = np.random.default_rng(38)
    hkv, n = 4, 1234
    k_tm = rand_bits(rng, n, hkv, D)
    ks = ts.chunk_key_sums(dev(k_tm).transpose(0, 1), 64)
    assert_close(ks.cpu().numpy(), C.chunk_key_sums(np.ascontiguousarray(k_tm.transpose(1, 0, 2)), 64), "key sums token-major")


def test_stream_read_probe_reads_every_vector(ts):
    """The measurement probe folds what it reads into a word that it stores only when the fold hits one
    value: a buffer of zeros leaves the sink alone, and planting that value anywhere (first vector,
    a middle one, the last one of a ragged tail) makes the owning thread store it."""
    import torch
    n_words = (3 * 32768 + 5 * 16) // 4            # three whole workgroup pieces and a ragged tail
    for where in (None, 0, n_words // 2 + 1, n_words - 1):
        buf = torch.zeros(n_words, dtype=torch.int32, device="cuda")
        if where is not None:
            buf[where] = 0x5CA1AB1E
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        ts.stream_read_probe(buf, sink)
        torch.cuda.synchronize()
        assert int(sink.item()) == (0 if where is None else 0x5CA1AB1E)
