"""Pins for the oracle's noise specification: the counter-based generator, the
integer inverse-CDF table of the discrete Gaussian (Def. 3.3) and the noisy
copy x + delta saturated to the 8-bit grid."""
import os

import mpmath as mp
import numpy as np
import pytest

import oracle


def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) if l[0] != "#" and l.strip()]
    assert len(rows) == 3
    for r in rows:
        v = [int(t, 16) for t in r]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(t) for t in out] == v[6:10]


def test_uniform64_counter_layout():
    """Pixel p reads word p&3 of the block with counter (p>>2, sample, image,
    phase*2+half); half 0 is the high word."""
    seed, image, phase, sample = 0x0123456789ABCDEF, 7, 1, 99999
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for p in (0, 1, 2, 3, 4, 150527, 3071):
        hi = oracle.philox4x32_10([p >> 2, sample, image, phase * 2 + 0], key)
        lo = oracle.philox4x32_10([p >> 2, sample, image, phase * 2 + 1], key)
        want = (int(hi[p & 3]) << 32) | int(lo[p & 3])
        assert oracle.uniform64(seed, image, phase, sample, p) == want
    # each field matters
    base = oracle.uniform64(1, 2, 0, 3, 40)
    assert len({base, oracle.uniform64(2, 2, 0, 3, 40), oracle.uniform64(1, 3, 0, 3, 40),
                oracle.uniform64(1, 2, 1, 3, 40), oracle.uniform64(1, 2, 0, 4, 40),
                oracle.uniform64(1, 2, 0, 3, 41), oracle.uniform64(1, 2, 0, 3, 44)}) == 7


def _exact_pmf(sigma, kmax):
    mp.mp.dps = 50
    w = [mp.e ** (-(mp.mpf(k) ** 2) / (2 * mp.mpf(sigma) ** 2)) for k in range(0, kmax + 400)]
    Z = w[0] + 2 * sum(w[1:])
    return [x / Z for x in w], Z


@pytest.mark.parametrize("sigma", [1, 2, 15, 32, 64, 128, 256])
def test_table_matches_closed_form_pmf(sigma):
    """Def. 3.3 with mu = 0: P[X = k] = exp(-k^2/2sigma^2) / sum_h exp(-h^2/2sigma^2).
    The table's cell widths must reproduce it to ~1e-15 and the support must
    leave out less than 1e-15 of the mass."""
    T, R = oracle.noise_table(sigma)
    assert len(T) == 2 * R
    t = [int(v) for v in T]
    assert all(b >= a for a, b in zip(t, t[1:]))
    assert 1 <= t[0] and t[-1] < 2 ** 64
    pmf, _ = _exact_pmf(sigma, R)
    two64 = mp.mpf(2) ** 64
    # cell k = -R is [0, T[0]); cell k in (-R, R) is [T[k+R-1], T[k+R]); cell R is [T[2R-1], 2^64)
    worst = mp.mpf(0)
    for k in range(-R, R + 1):
        lo = 0 if k == -R else t[k + R - 1]
        hi = 2 ** 64 if k == R else t[k + R]
        worst = max(worst, abs(mp.mpf(hi - lo) / two64 - pmf[abs(k)]))
    assert worst < mp.mpf("3e-15")
    tail = 2 * sum(pmf[R + 1:])
    assert tail < mp.mpf("1e-15")
    # symmetry of the law: P[X <= -1] = P[X >= 1]
    assert abs(t[R - 1] - (2 ** 64 - t[R])) <= 2


def test_table_moments_closed_form():
    """Mean 0 and variance of the table law vs the exact discrete-Gaussian variance."""
    for sigma in (2, 32, 128):
        T, R = oracle.noise_table(sigma)
        t = [0] + [int(v) for v in T] + [2 ** 64]
        pk = [(t[i + 1] - t[i]) for i in range(2 * R + 1)]  # integer masses / 2^64
        mean = sum((i - R) * p for i, p in enumerate(pk)) / 2.0 ** 64
        var = sum((i - R) ** 2 * p for i, p in enumerate(pk)) / 2.0 ** 64
        pmf, _ = _exact_pmf(sigma, R)
        var_exact = 2 * sum(mp.mpf(k) ** 2 * pmf[k] for k in range(1, len(pmf)))
        assert abs(mean) < 1e-12
        assert abs(var - float(var_exact)) / float(var_exact) < 1e-12
        assert abs(var / sigma ** 2 - 1) < 1e-6


@pytest.mark.parametrize("sigma", [1, 32, 256])
def test_delta_is_inverse_cdf(sigma):
    """delta(u) is the smallest k with u/2^64 < P[X <= k] (exact 50-digit cdf),
    away from cell boundaries."""
    T, R = oracle.noise_table(sigma)
    pmf, _ = _exact_pmf(sigma, R)
    mp.mp.dps = 50
    ks = list(range(-R - 300, R + 301))
    cdf, acc = [], mp.mpf(0)
    for k in ks:
        acc += pmf[abs(k)] if abs(k) < len(pmf) else 0
        cdf.append(acc)
    rng = np.random.default_rng(5)
    us = [int(v) for v in rng.integers(0, 2 ** 64, size=300, dtype=np.uint64)]
    us += [0, 2 ** 64 - 1, 2 ** 63, 2 ** 63 - 1, 12345, 2 ** 64 - 98765]
    checked = 0
    for u in us:
        x = mp.mpf(u) / mp.mpf(2) ** 64
        idx = next(i for i, c in enumerate(cdf) if x < c)
        near = min(abs(cdf[idx] - x), abs(x - cdf[idx - 1]) if idx else 1)
        got = oracle.delta(T, R, u)
        if near > mp.mpf("1e-14"):
            assert got == ks[idx], (u, got, ks[idx])
            checked += 1
        else:  # boundary case: tail cells narrower than the table's resolution
            assert abs(got - ks[idx]) <= 300
    assert checked >= 295
    assert oracle.delta(T, R, 0) == -R and oracle.delta(T, R, 2 ** 64 - 1) == R


def test_delta_worked_examples():
    """First block of the stream (seed 0, image 0, phase 0, sample 0): the high
    words are the all-zero known answer; delta follows from the inverse cdf of
    N(0, sigma^2) up to the half-integer continuity correction."""
    hi = [0x6627E8D5, 0xE169C58D, 0xBC57AC4C, 0x9B00DBD8]
    for p in range(4):
        assert oracle.uniform64(0, 0, 0, 0, p) >> 32 == hi[p]
    mp.mp.dps = 30
    for sigma in (32, 64, 128, 256):
        T, R = oracle.noise_table(sigma)
        for p in range(4):
            u = oracle.uniform64(0, 0, 0, 0, p)
            z = mp.sqrt(2) * mp.erfinv(2 * mp.mpf(u) / mp.mpf(2) ** 64 - 1) * sigma
            assert abs(oracle.delta(T, R, u) - float(z)) <= 0.5 + 1e-3 * sigma


def test_sampler_empirical_law():
    """Empirical mean, variance, kurtosis, E|delta| and a chi-square of draws
    from the stream against the closed-form law."""
    sigma = 32
    T, R = oracle.noise_table(sigma)
    n = 200000
    d = np.array([oracle.delta(T, R, oracle.uniform64(11, 3, 1, 5, p)) for p in range(n)], dtype=np.float64)
    assert abs(d.mean()) < 4 * sigma / np.sqrt(n)
    assert abs(d.var() / sigma ** 2 - 1) < 0.02
    assert abs(((d - d.mean()) ** 4).mean() / d.var() ** 2 - 3) < 0.08
    assert abs(np.abs(d).mean() / sigma - 0.797819626) < 0.01
    pmf, _ = _exact_pmf(sigma, R)
    edges = list(range(-96, 97, 8))
    obs = np.histogram(d, bins=[-1e9] + [e - 0.5 for e in edges] + [1e9])[0]
    probs = []
    lo = -10 ** 6
    for e in edges + [10 ** 6]:
        probs.append(float(sum(pmf[abs(k)] for k in range(max(lo, -R - 300), min(e, R + 301)))))
        lo = e
    exp = np.array(probs) * n
    chi2 = ((obs - exp) ** 2 / exp).sum()
    assert chi2 < 60.0  # 25 dof: P[chi2 > 60] ~ 1e-4


def test_noisy_copy_clamps_and_recentres():
    sigma = 64
    T, R = oracle.noise_table(sigma)
    x = np.zeros((3, 8, 8), dtype=np.uint8)
    x[1] = 255
    x[2] = 100
    a0 = oracle.noisy(x, sigma, 9, 4, 1, 17)
    assert a0.dtype == np.int8 and a0.shape == x.shape
    flat = x.reshape(-1)
    for p in range(flat.size):
        d = oracle.delta(T, R, oracle.uniform64(9, 4, 1, 17, p))
        want = min(255, max(0, int(flat[p]) + d)) - 128
        assert int(a0.reshape(-1)[p]) == want
    assert (a0[0] == -128).mean() > 0.3   # about half the draws are <= 0
    assert (a0[1] == 127).mean() > 0.3


def test_table_argument_domain():
    with pytest.raises(ValueError):
        oracle.noise_table(0)
    with pytest.raises(ValueError):
        oracle.noise_table(1025)
    T, R = oracle.noise_table(1024)
    assert len(T) == 2 * R


def test_noise_bank_counter_layout_and_range():
    """Stored training noise: tensor index in the sample word, bank id in the image word,
    phase 2 (counter word 4 | half), unsaturated draws.  Checked through the Philox routine
    (pinned above by known answers) and a sorted-table lookup."""
    sigma, seed, bank, first, count, d = 256, 0xFEDCBA9876543210, 5, 1000, 3, 64
    T, R = oracle.noise_table(sigma)
    got = oracle.noise_bank(sigma, seed, bank, first, count, d)
    assert got.shape == (count, d) and got.dtype == np.int16
    key = [seed & 0xFFFFFFFF, seed >> 32]
    for t in range(count):
        for p in range(d):
            hi = oracle.philox4x32_10([p >> 2, first + t, bank, 4], key)
            lo = oracle.philox4x32_10([p >> 2, first + t, bank, 5], key)
            u = (int(hi[p & 3]) << 32) | int(lo[p & 3])
            assert int(got[t, p]) == int(np.searchsorted(T, np.uint64(u), side="right")) - R
    assert np.abs(got).max() > 255            # nothing saturates at the pixel range
    # disjoint from the inference streams (phases 0 and 1) and from other banks / tensors
    for phase in (0, 1):
        other = np.array([oracle.delta(T, R, oracle.uniform64(seed, bank, phase, first, p)) for p in range(d)])
        assert not np.array_equal(other, got[0])
    assert not np.array_equal(oracle.noise_bank(sigma, seed, bank + 1, first, 1, d)[0], got[0])
    assert not np.array_equal(got[0], got[1])
    # a range of tensors is reproducible piecewise
    assert np.array_equal(oracle.noise_bank(sigma, seed, bank, first + 1, 2, d), got[1:])


@pytest.mark.parametrize("sigma", [2, 32])
def test_noise_bank_empirical_law(sigma):
    """Mean 0, variance sigma^2 and a chi-square of a stored bank against Def. 3.3."""
    T, R = oracle.noise_table(sigma)
    bank = oracle.noise_bank(sigma, 7, 1, 0, 64, 3072).astype(np.float64).reshape(-1)
    n = bank.size
    assert abs(bank.mean()) < 4 * sigma / np.sqrt(n)
    assert abs(bank.var() / sigma ** 2 - 1) < 0.02
    pmf, _ = _exact_pmf(sigma, R)
    step = max(1, sigma // 4)
    edges = list(range(-3 * sigma, 3 * sigma + 1, step))
    obs = np.histogram(bank, bins=[-1e9] + [e - 0.5 for e in edges] + [1e9])[0]
    probs, lo = [], -10 ** 6
    for e in edges + [10 ** 6]:
        probs.append(float(sum(pmf[abs(k)] for k in range(max(lo, -R - 300), min(e, R + 301)))))
        lo = e
    exp = np.array(probs) * n
    chi2 = ((obs - exp) ** 2 / exp).sum()
    assert chi2 < 70.0   # 25 degrees of freedom: P[chi2 > 70] ~ 4e-6
