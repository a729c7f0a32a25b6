"""CPU oracle for the penalized sampling step -- TEST INFRASTRUCTURE ONLY.

Plain numpy in float64; shares nothing with the GPU library.  Passages followed:
  penalized_probs   Sec. 3.4 "Contextual Penalty", Eq. 3: softmax of l_i / (t * I_i) with I_i = theta for
                    tokens that occur among the W most recent generated tokens and 1 otherwise.
  pool_threshold    App. D: the sampling pools of min-p (probability >= p_base * p_max), top-p (the most
                    probable tokens whose mass reaches p) and eta-sampling (probability >= min(epsilon,
                    alpha * exp(-entropy))), all written as "probability >= tau".
  sample            App. D: the next token is drawn from the pool with the renormalised probabilities;
                    here by inverting the pool's cumulative distribution, taken in order of token id,
                    at a uniform number that is passed in.
Pins: tests/test_sampling_pins.py.
"""
import numpy as np

FULL, MIN_P, TOP_P, ETA = 0, 1, 2, 3


def penalized_probs(logits, window, temperature, theta):
    """logits [R, V] (any float dtype, widened), window: iterable of token ids -> float64 [R, V]."""
    l = np.asarray(logits, dtype=np.float64)
    indicator = np.ones(l.shape[1], dtype=np.float64)
    for tok in window:
        indicator[int(tok)] = theta
    x = l / (temperature * indicator)
    x = x - x.max(axis=1, keepdims=True)
    e = np.exp(x)
    return e / e.sum(axis=1, keepdims=True)


def pool_threshold(p_row, method, param, param2=0.0):
    """Probability threshold tau of the pool {v : p[v] >= tau} for one row, in float64 (the row is widened
    exactly; the result is a Python float)."""
    p = np.asarray(p_row, dtype=np.float64)
    if method == FULL:
        return 0.0
    if method == MIN_P:
        return float(param) * float(p.max())
    if method == TOP_P:
        # smallest set of most probable tokens whose mass reaches `param`: walk the tokens in order of
        # decreasing probability; tokens tied with the last one taken are all kept
        order = np.argsort(-p, kind="stable")
        mass = 0.0
        tau = float(p[order[-1]])
        for v in order:
            mass += float(p[v])
            if mass >= param:
                tau = float(p[v])
                break
        return tau
    if method == ETA:
        # eta = min(epsilon, alpha * exp(-h)), h = entropy of the row (natural log); param = epsilon, param2 = alpha
        h = -float(np.sum(np.where(p > 0, p * np.log(np.where(p > 0, p, 1.0)), 0.0)))
        return min(float(param), float(param2) * float(np.exp(-h)))
    raise ValueError(method)


def sample_from_pool(p_row, tau, u):
    """Draw from the pool {v : p[v] >= tau} with the renormalised probabilities, by inverting the pool's
    cumulative distribution (taken in order of token id) at u.
    -> (token, pool_mass, margin): margin = distance of u*pool_mass to the nearest step of that
    cumulative distribution, relative to pool_mass (how decisive the draw was)."""
    p = np.asarray(p_row, dtype=np.float64)
    in_pool = p >= float(tau)
    w = np.where(in_pool, p, 0.0)
    cdf = np.cumsum(w)
    mass = cdf[-1]
    target = float(u) * mass
    tok = int(np.searchsorted(cdf, target, side="right"))     # first id whose cumulative mass exceeds the target
    tok = min(tok, int(np.nonzero(in_pool)[0][-1]))
    steps = cdf[in_pool]
    margin = float(np.min(np.abs(steps - target))) / mass
    return tok, mass, margin


def sample(p_row, method, param, u, param2=0.0):
    """-> (token, pool_mass, margin) for the pool of `method` (see pool_threshold and sample_from_pool)."""
    return sample_from_pool(p_row, pool_threshold(p_row, method, param, param2), u)
