"""GPU parity of the penalized probabilities and the pool sampler (through the C ABI) against the
numpy oracle.  Probabilities: the floating-point bar.  Pool thresholds and sampled tokens are
decisions that floating point takes.  The oracle (fp64) is given the GPU's own fp32 probabilities; the
test states, from the oracle's side, which thresholds are admissible given fp32 rounding and requires
the GPU's to be one of them; the draw is then compared exactly with the oracle's draw from the pool of
that threshold, unless the oracle says the draw was not decisive (the target within 1e-5 of a step of
the cumulative distribution), in which case the neighbouring pool token is accepted as well."""
import numpy as np
import pytest

from oracle import sampling as O
from gpu_util import assert_close

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ts():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    import paper_2502_18890_amd as lib
    lib.load_library()
    return lib


def _logits(rng, r, v, spread=3.0):
    return (rng.standard_normal((r, v)) * spread).astype(np.float32)


@pytest.mark.parametrize("r,v,nw,t,theta", [(4, 1000, 16, 1.0, 1.2), (3, 4096, 100, 0.7, 1.15), (2, 4097, 0, 1.3, 1.5),
                                            (5, 32000, 1024, 1.0, 1.15), (2, 128256, 1024, 1.0, 1.2), (1, 151936, 2048, 0.9, 1.13),
                                            (7, 33, 5, 1.0, 2.0), (1, 1, 1, 1.0, 1.2)])
def test_penalized_probs(ts, r, v, nw, t, theta):
    import torch
    rng = np.random.default_rng(41)
    lg = _logits(rng, r, v)
    window = rng.integers(0, v, size=nw).astype(np.int32)
    if nw > 3:
        window[1] = window[0]                   # repeats are allowed
    got = ts.penalized_probs(torch.from_numpy(lg).cuda(), torch.from_numpy(window).cuda() if nw else None, t, theta)
    ref = O.penalized_probs(lg, window, t, theta)
    assert_close(got.cpu().numpy(), ref, "penalized probs")
    np.testing.assert_allclose(got.cpu().numpy().astype(np.float64).sum(axis=1), 1.0, rtol=0, atol=1e-5)


def test_penalized_probs_peaked_and_flat_rows(ts):
    import torch
    v = 5000
    lg = np.zeros((3, v), dtype=np.float32)
    lg[0, 77] = 60.0                            # one token takes everything
    lg[1, :] = -200.0                           # flat and far from zero
    lg[2, ::2] = 30.0
    window = np.array([77, 78, 0], dtype=np.int32)
    got = ts.penalized_probs(torch.from_numpy(lg).cuda(), torch.from_numpy(window).cuda(), 1.0, 1.2).cpu().numpy()
    assert_close(got, O.penalized_probs(lg, window, 1.0, 1.2), "penalized probs, peaked/flat")


def _pool_mass(p64, tau):
    return float(p64[p64 >= tau].sum())


def _assert_threshold_admissible(p_row, method, param, param2, thr):
    """The threshold is a decision floating point takes.  The admissible thresholds are stated here from the
    oracle's side (fp64 on the row's exact values), and the GPU's must be one of them:
      full   tau = 0.
      min-p  tau = p_base * p_max up to fp32 rounding; the pool may differ from the oracle's only in tokens whose
             probability lies within that rounding of the threshold.
      top-p  the pool {p >= tau} holds mass >= p - 1e-6 (or is the whole row), and without its least probable members
             (the tokens tied at its minimum) it holds mass < p + 1e-6: the smallest pool that reaches p,
             where masses within 1e-6 of p count as either side (the kernel adds masses in units of 2^-40, each
             probability within half a unit: 7e-8 over a vocabulary of 152K).
      eta    tau = min(epsilon, alpha * exp(-entropy)) to 2e-5 relative (an fp32 sum over the vocabulary); the pool may
             differ from the oracle's only in tokens within that distance of the threshold."""
    p64 = np.asarray(p_row, dtype=np.float64)
    thr = float(thr)
    tau = O.pool_threshold(p_row, method, float(np.float32(param)), float(np.float32(param2)))
    if method == O.FULL:
        assert thr == 0.0
        return
    if method == O.TOP_P:
        if thr == tau:
            return
        want = float(np.float32(param))
        pool = p64[p64 >= thr]
        assert pool.size > 0, ("top-p pool is empty", thr)
        # it reaches p -- or it is the whole row, when even that falls short of p (p = 1 and a row that sums to 1 - 1e-7)
        assert float(pool.sum()) >= want - 1e-6 or pool.size == p64.size, ("top-p pool too small", thr, float(pool.sum()), want)
        # and it is minimal: without its least probable members (all tied at the pool's minimum) it does not reach p
        assert _pool_mass(p64, float(np.nextafter(pool.min(), np.inf))) < want + 1e-6, ("top-p pool not minimal", thr, tau)
        return
    rel = 1e-6 if method == O.MIN_P else 2e-5
    assert abs(thr - tau) <= rel * tau, (method, thr, tau)
    differs = (p64 >= thr) != (p64 >= tau)
    assert np.all(np.abs(p64[differs] - tau) <= rel * tau), ("pool differs away from the threshold", method, thr, tau)


def _check_draws(ts, probs_gpu, method, param, u, param2=0.0):
    import torch
    p = probs_gpu.cpu().numpy()
    tok, thr, mass = ts.sample_tokens(probs_gpu, method, param, torch.from_numpy(u).cuda(), want_pool=True, param2=param2)
    tok, thr, mass = tok.cpu().numpy(), thr.cpu().numpy(), mass.cpu().numpy()
    n_ambiguous = 0
    for r in range(p.shape[0]):
        _assert_threshold_admissible(p[r], method, param, param2, thr[r])
        # the draw, against the pool the oracle derives from that (admissible) threshold
        ref_tok, ref_mass, margin = O.sample_from_pool(p[r], float(thr[r]), u[r])
        assert abs(mass[r] - ref_mass) <= 1e-5 * max(ref_mass, 1e-30)
        assert p[r, tok[r]] >= thr[r] and p[r, tok[r]] > 0
        if tok[r] != ref_tok:
            assert margin < 1e-5, (r, tok[r], ref_tok, margin)
            pool_ids = np.nonzero(p[r] >= thr[r])[0]
            assert abs(int(np.searchsorted(pool_ids, tok[r])) - int(np.searchsorted(pool_ids, ref_tok))) == 1
            n_ambiguous += 1
    assert n_ambiguous <= max(1, p.shape[0] // 10)


@pytest.mark.parametrize("method,param", [(O.FULL, 0.0), (O.MIN_P, 0.1), (O.MIN_P, 0.05), (O.MIN_P, 1.0), (O.TOP_P, 0.9), (O.TOP_P, 0.5),
                                          (O.TOP_P, 1.0)])
@pytest.mark.parametrize("r,v", [(40, 1000), (16, 32000), (8, 128256), (3, 4099)])
def test_sampling_pools_and_draws(ts, method, param, r, v):
    import torch
    rng = np.random.default_rng(42)
    lg = _logits(rng, r, v, spread=2.5)
    probs = ts.penalized_probs(torch.from_numpy(lg).cuda(), None, 1.0, 1.0)
    u = rng.random(r).astype(np.float32)
    u[0] = 0.0
    u[-1] = 0.99999
    _check_draws(ts, probs, method, param, u)


@pytest.mark.parametrize("eps,alpha", [(0.0009, 0.03), (0.3, 0.5), (1.0, 5.0)])
@pytest.mark.parametrize("r,v", [(24, 1000), (6, 128256)])
def test_eta_sampling(ts, eps, alpha, r, v):
    import torch
    rng = np.random.default_rng(43)
    lg = _logits(rng, r, v, spread=2.0)
    probs = ts.penalized_probs(torch.from_numpy(lg).cuda(), None, 1.0, 1.0)
    _check_draws(ts, probs, O.ETA, eps, rng.random(r).astype(np.float32), param2=alpha)


def test_sampling_with_ties_and_tiny_vocab(ts):
    import torch
    p = np.array([[0.3, 0.2, 0.2, 0.2, 0.1], [0.0, 0.5, 0.0, 0.5, 0.0], [1.0, 0.0, 0.0, 0.0, 0.0]], dtype=np.float32)
    pg = torch.from_numpy(p).cuda()
    for method, param in ((O.TOP_P, 0.45), (O.MIN_P, 0.6), (O.FULL, 0.0)):
        for uu in (0.0, 0.31, 0.5, 0.77, 0.99):
            _check_draws(ts, pg, method, param, np.full(3, uu, dtype=np.float32))


def test_sampling_frequencies_follow_the_pool_distribution(ts):
    """Many rows with the same distribution and a grid of uniforms: token counts match the
    renormalised pool probabilities."""
    import torch
    base = np.array([0.02, 0.38, 0.1, 0.25, 0.2, 0.05], dtype=np.float32)
    n = 4000
    pg = torch.from_numpy(np.tile(base, (n, 1))).cuda()
    u = ((np.arange(n) + 0.5) / n).astype(np.float32)
    for method, param in ((O.MIN_P, 0.3), (O.TOP_P, 0.8)):
        tok = ts.sample_tokens(pg, method, param, torch.from_numpy(u).cuda()).cpu().numpy()
        tau = O.pool_threshold(base, method, param)
        want = np.where(base >= tau, base, 0.0).astype(np.float64)
        want /= want.sum()
        np.testing.assert_allclose(np.bincount(tok, minlength=6) / n, want, rtol=0, atol=2.0 / n)


def test_top_p_edge_rows_and_repeatability(ts):
    """Rows that stress the digit-by-digit threshold search: one dominant token, a long tail of tiny and
    subnormal probabilities, many equal values around the cut, zeros; the same call twice gives the same
    tokens, thresholds and masses bit for bit."""
    import torch
    rng = np.random.default_rng(7)
    v = 20000
    rows = []
    a = np.full(v, 1e-30, dtype=np.float64); a[123] = 1.0; rows.append(a)                       # dominant token
    b = rng.random(v) ** 12; b[::3] = 0.0; rows.append(b)                                       # heavy tail + zeros
    c = np.full(v, 1.0); c[:50] = 40.0; rows.append(c)                                          # plateau: ties at the cut
    d = np.exp(rng.normal(0, 6.0, v)); d[5] = 1e-44; d[6] = 3e-39; rows.append(d)               # subnormals present
    e = np.zeros(v); e[[7, 19999]] = 0.5; rows.append(e)                                        # two tokens, rest zero
    p = np.stack([r / r.sum() for r in rows]).astype(np.float32)
    pg = torch.from_numpy(p).cuda()
    u = np.array([0.3, 0.999, 0.5, 0.01, 0.75], dtype=np.float32)
    for param in (0.05, 0.5, 0.9, 0.999):
        _check_draws(ts, pg, O.TOP_P, param, u)
        first = [x.cpu().numpy() for x in ts.sample_tokens(pg, O.TOP_P, param, torch.from_numpy(u).cuda(), want_pool=True)]
        again = [x.cpu().numpy() for x in ts.sample_tokens(pg, O.TOP_P, param, torch.from_numpy(u).cuda(), want_pool=True)]
        for x, y in zip(first, again):
            assert x.tobytes() == y.tobytes()
