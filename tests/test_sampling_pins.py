"""Pins of the sampling oracle (CPU only): Eq. 3 and the pools of App. D against closed forms, library
routines and brute force."""
import numpy as np
import pytest
from scipy.special import softmax

from oracle import sampling as O


def test_no_penalty_is_plain_temperature_softmax():
    rng = np.random.default_rng(1)
    l = rng.standard_normal((5, 300)) * 3
    for t in (1.0, 0.7, 1.9):
        np.testing.assert_allclose(O.penalized_probs(l, [], t, 1.2), softmax(l / t, axis=1), rtol=0, atol=1e-15)
        np.testing.assert_allclose(O.penalized_probs(l, [3, 7, 7, 299], t, 1.0), softmax(l / t, axis=1), rtol=0, atol=1e-15)


def test_penalty_closed_form_ratios_and_normalisation():
    """Eq. 3: for i in the window and j outside, p_i / p_j = exp(l_i/(t theta) - l_j/t); rows sum to 1."""
    rng = np.random.default_rng(2)
    l = rng.standard_normal((3, 50)) * 4
    window, t, theta = [4, 9, 9, 30], 0.8, 1.15
    p = O.penalized_probs(l, window, t, theta)
    np.testing.assert_allclose(p.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    for r in range(3):
        for i in (4, 9, 30):
            for j in (0, 10, 49):
                assert np.isclose(p[r, i] / p[r, j], np.exp(l[r, i] / (t * theta) - l[r, j] / t), rtol=1e-12)
        assert np.isclose(p[r, 4] / p[r, 30], np.exp((l[r, 4] - l[r, 30]) / (t * theta)), rtol=1e-12)   # both penalised
    # the printed formula divides the logit: a positive logit in the window loses mass, a negative one gains
    l2 = np.array([[2.0, -2.0, 0.5, 0.1]])
    base = O.penalized_probs(l2, [], 1.0, 1.2)
    assert O.penalized_probs(l2, [0], 1.0, 1.2)[0, 0] < base[0, 0]
    assert O.penalized_probs(l2, [1], 1.0, 1.2)[0, 1] > base[0, 1]


def test_two_token_logistic():
    # V = 2, token 0 penalised: p_0 = 1 / (1 + exp(l_1/t - l_0/(t theta)))
    l = np.array([[1.3, -0.4]])
    p = O.penalized_probs(l, [0], 0.5, 1.2)
    assert np.isclose(p[0, 0], 1.0 / (1.0 + np.exp(-0.4 / 0.5 - 1.3 / (0.5 * 1.2))), rtol=1e-14)


def test_min_p_pool_brute_force():
    rng = np.random.default_rng(3)
    p = softmax(rng.standard_normal(200) * 2)
    for p_base in (0.05, 0.1, 0.5, 1.0):
        tau = O.pool_threshold(p, O.MIN_P, p_base)
        pool = {v for v in range(200) if p[v] >= p_base * max(p)}
        assert {v for v in range(200) if p[v] >= tau} == pool
    assert {v for v in range(200) if p[v] >= O.pool_threshold(p, O.MIN_P, 1.0)} == {int(np.argmax(p))}
    assert O.pool_threshold(p, O.FULL, 0.0) == 0


def test_top_p_pool_is_the_smallest_prefix_of_the_sorted_tokens():
    p = np.array([0.05, 0.4, 0.1, 0.25, 0.2])              # sorted: 0.4 0.25 0.2 0.1 0.05
    pools = {0.3: {1}, 0.4: {1}, 0.41: {1, 3}, 0.65: {1, 3}, 0.66: {1, 3, 4}, 0.9: {1, 3, 4, 2}, 1.0: {0, 1, 2, 3, 4}}
    for pp, want in pools.items():
        tau = O.pool_threshold(p, O.TOP_P, pp)
        assert {v for v in range(5) if p[v] >= tau} == want, pp
    # brute force on random rows: removing the least probable pool member must drop the mass below p
    rng = np.random.default_rng(4)
    for _ in range(20):
        q = softmax(rng.standard_normal(64) * 2)
        tau = O.pool_threshold(q, O.TOP_P, 0.9)
        pool = q[q >= tau]
        assert pool.sum() >= 0.9 and pool.sum() - pool.min() < 0.9
        assert q[q < tau].max(initial=0.0) <= pool.min()


def test_eta_pool_closed_forms():
    # uniform row over n tokens: entropy = log n, so alpha * exp(-h) = alpha / n
    n = 50
    p = np.full(n, 1.0 / n)
    assert np.isclose(O.pool_threshold(p, O.ETA, 0.5, 2.0), 2.0 / n)          # alpha/n < epsilon
    assert np.isclose(O.pool_threshold(p, O.ETA, 0.001, 2.0), 0.001)         # epsilon caps it
    # one-hot row: entropy 0, eta = min(epsilon, alpha); pool = the hot token when eta <= 1
    hot = np.zeros(10); hot[3] = 1.0
    tau = O.pool_threshold(hot, O.ETA, 0.9, 0.5)
    assert np.isclose(tau, 0.5) and {v for v in range(10) if hot[v] >= tau} == {3}
    # two tokens (a, 1-a): entropy by the textbook formula
    a = 0.2
    h = -(a * np.log(a) + (1 - a) * np.log(1 - a))
    assert np.isclose(O.pool_threshold(np.array([a, 1 - a]), O.ETA, 1.0, 0.3), 0.3 * np.exp(-h))
    from scipy.stats import entropy
    rng = np.random.default_rng(7)
    q = softmax(rng.standard_normal(300) * 2)
    assert np.isclose(O.pool_threshold(q, O.ETA, 1.0, 0.7), 0.7 * np.exp(-entropy(q)))


def test_ties_at_the_cut_are_kept_together():
    p = np.array([0.3, 0.2, 0.2, 0.2, 0.1])
    tau = O.pool_threshold(p, O.TOP_P, 0.45)               # 0.3 + one of the 0.2s reaches 0.45: all three 0.2s stay
    assert {v for v in range(5) if p[v] >= tau} == {0, 1, 2, 3}


def test_sampling_inverts_the_renormalised_pool_distribution():
    """Over a fine grid of uniforms, token frequencies equal the renormalised pool probabilities."""
    p = np.array([0.02, 0.38, 0.1, 0.25, 0.2, 0.05])
    for method, param in ((O.FULL, 0.0), (O.MIN_P, 0.3), (O.TOP_P, 0.8)):
        tau = O.pool_threshold(p, method, param)
        want = np.where(p >= tau, p, 0.0)
        want = want / want.sum()
        n = 20000
        counts = np.zeros(6)
        for i in range(n):
            tok, mass, _ = O.sample(p, method, param, (i + 0.5) / n)
            counts[tok] += 1
        np.testing.assert_allclose(counts / n, want, rtol=0, atol=1.5 / n)
        assert np.isclose(mass, p[p >= tau].sum())
    # u = 0 gives the first pool token, u -> 1 the last
    assert O.sample(p, O.MIN_P, 0.3, 0.0)[0] == 1 and O.sample(p, O.MIN_P, 0.3, 0.999999)[0] == 4
