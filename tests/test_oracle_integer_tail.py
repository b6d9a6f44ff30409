"""Pins of the oracle's integer-only certification tail (Thm 3.2, proof steps 2-3):
the discrete-Gaussian quantile by table lookup against the cdf summed directly from
Def. 3.3 in 60-digit arithmetic, against the normal quantile it must approach, and
against the symmetry and monotonicity the definition fixes."""
import math

import mpmath as mp
import numpy as np
import pytest

from oracle import stats

mp.mp.dps = 60


def _exact_cdf(sigma, lo, hi):
    """{t: P[delta <= t]} for t in [lo, hi], pmf proportional to exp(-k^2 / (2 sigma^2)) over Z."""
    K = int(14 * sigma) + 20
    w = {k: mp.e ** (-mp.mpf(k * k) / (2 * sigma * sigma)) for k in range(-K, K + 1)}
    tot = mp.fsum(w.values())
    acc = mp.fsum(w[k] for k in range(-K, lo))
    out = {}
    for t in range(lo, hi + 1):
        acc += w[t]
        out[t] = acc / tot
    return out


@pytest.mark.parametrize("sigma", [1, 4, 32, 64, 256])
def test_quantile_is_the_largest_point_with_cdf_at_most_p(sigma):
    span = int(6 * sigma) + 2
    cdf = _exact_cdf(sigma, -span, span)
    rng = np.random.default_rng(sigma)
    ps = list(rng.uniform(0.5, 1.0, 40)) + [0.5, 0.75, 0.9, 0.99, 0.999, 0.999999, 1 - 1e-9]
    checked = 0
    for p in ps:
        want = max((t for t in cdf if cdf[t] <= mp.mpf(p)), default=None)
        if want is None or want >= span:
            continue
        # skip levels closer than the table's 2^-60 resolution to a cdf value
        if min(abs(cdf[want] - p), abs(cdf[want + 1] - p)) < mp.mpf(2) ** -58:
            continue
        assert stats.discrete_quantile(sigma, float(p)) == want, (sigma, p)
        checked += 1
    assert checked > 30


@pytest.mark.parametrize("sigma", [32, 64, 128, 256, 1024])
def test_quantile_approaches_the_normal_one(sigma):
    """For sigma >= 32 the lattice cdf at t equals the normal cdf at (t + 1/2) / sigma to
    well under 1e-6 (Euler-Maclaurin), so the lookup lands within one grid unit of
    sigma * Phi^-1(p) - 1/2, the quantity Alg. 1 prints."""
    for p in (0.5001, 0.6, 0.75, 0.9, 0.99, 0.9999, 1 - 1e-7):
        t = stats.discrete_quantile(sigma, p)
        cont = stats.radius(sigma, p)
        assert cont - 1.5 - 1e-6 <= t <= cont - 0.5 + 1e-6 + 1e-3 * sigma * (p > 0.99999), (sigma, p, t, cont)


def test_symmetry_and_monotonicity_and_edges():
    for sigma in (3, 32, 100):
        prev = -10 ** 9
        for p in np.linspace(0.01, 0.99, 99):
            t = stats.discrete_quantile(sigma, float(p))
            assert t >= prev
            prev = t
        # P[delta <= t] + P[delta <= -t - 1] = 1: quantiles of p and 1 - p mirror around -1/2
        for p in (0.6, 0.8, 0.95):
            a, b = stats.discrete_quantile(sigma, p), stats.discrete_quantile(sigma, 1 - p)
            assert a + b in (-2, -1), (sigma, p, a, b)
        # at most one half the quantile is negative: nothing is certified
        assert stats.discrete_quantile(sigma, 0.5) == -1
        assert stats.radius_squared_int(sigma, 0.5) == 0 and stats.radius_squared_int(sigma, 0.3) == 0
        t = stats.discrete_quantile(sigma, 0.9)
        assert stats.radius_squared_int(sigma, 0.9) == t * t and t > 0
    # p = 1: every table entry is below 2^64, the last lattice point before the support's end (R = 271)
    assert stats.discrete_quantile(32, 1.0) == 270 and stats.discrete_quantile(32, 0.0) == -272
    with pytest.raises(ValueError):
        stats.discrete_quantile(32, 1.5)


def test_integer_certification_on_hand_tallies():
    """Alg. 1 with the integer tail (Thm 3.2, proof steps 2-3) on tallies whose outcome is fixed by
    the definitions: every estimation vote on one class gives p_A = alpha^(1/n), whose quantile
    under the lattice law is read here off the cdf summed from Def. 3.3 in 60 digits; a bound
    below one half abstains; the class comes from the selection tally, not the estimation tally."""
    sigma, n, alpha = 64, 1000, 0.001
    c0 = np.array([3, 90, 7], dtype=np.uint32)
    c1 = np.array([0, n, 0], dtype=np.uint32)
    cls, t, t2 = stats.certify_decision_integer(c0, c1, sigma, n, alpha)
    p = mp.mpf(alpha) ** (mp.mpf(1) / n)
    cdf = _exact_cdf(sigma, 100, 200)
    want = max(k for k in cdf if cdf[k] <= p)
    assert (cls, t, t2) == (1, want, want * want) and 100 < want < 200
    assert stats.radius(sigma, float(p)) - 1.5 <= t <= stats.radius(sigma, float(p)) - 0.5
    # the estimation tally's own top class is ignored: class 1 was selected, its 400 of 1000 votes abstain
    c1b = np.array([600, 400, 0], dtype=np.uint32)
    assert stats.certify_decision_integer(c0, c1b, sigma, n, alpha) == (stats.ABSTAIN, 0, 0)
    # selected class with 600 of 1000: p_A = 0.5510754739370525 (golden file), a small positive radius
    c1c = np.array([400, 600, 0], dtype=np.uint32)
    cls, t, t2 = stats.certify_decision_integer(c0, c1c, sigma, n, alpha)
    cdf = _exact_cdf(sigma, 0, 20)
    want = max(k for k in cdf if cdf[k] <= mp.mpf("0.55107547393705244475"))
    assert (cls, t, t2) == (1, want, want * want) and want == 7   # 64 * 0.12838 - 1/2 = 7.7
    # a bound just above one half: class returned, quantile -1 or 0, squared radius 0
    c1d = np.array([450, 550, 0], dtype=np.uint32)    # p_A = 0.50067596 (smallest certifying count)
    cls, t, t2 = stats.certify_decision_integer(c0, c1d, sigma, n, alpha)
    assert cls == 1 and t in (-1, 0) and t2 == 0
