"""Pins for the oracle's host statistics (Alg. 1 and Alg. 2 decisions)."""
import math
import os
from fractions import Fraction

import mpmath as mp
import numpy as np
import pytest

from oracle import stats

ALPHA = 0.001


def _golden(golden_dir):
    rows = []
    for l in open(os.path.join(golden_dir, "cp_radius_values.txt")):
        if l.startswith("#") or not l.strip():
            continue
        n, k, p, r = l.split()
        rows.append((int(n), int(k), p, r))
    return rows


def test_cp_lower_closed_forms():
    for n in (1, 10, 100, 1000, 100000):
        assert stats.cp_lower(0, n, ALPHA) == 0.0
        assert stats.cp_lower(n, n, ALPHA) == pytest.approx(ALPHA ** (1.0 / n), rel=1e-14)
    # k = 1: 1 - (1-p)^n = alpha
    for n in (5, 100, 100000):
        assert stats.cp_lower(1, n, ALPHA) == pytest.approx(-math.expm1(math.log1p(-ALPHA) / n), rel=1e-12)


@pytest.mark.parametrize("n,k", [(20, 13), (100, 66), (100, 30), (257, 200)])
def test_cp_lower_solves_exact_binomial_tail(n, k):
    """Brute force with exact rationals: the tail probability at the returned p
    equals alpha, and it is increasing in p."""
    p = Fraction(stats.cp_lower(k, n, ALPHA))

    def tail(q):
        return sum(math.comb(n, j) * q ** j * (1 - q) ** (n - j) for j in range(k, n + 1))

    t = tail(p)
    assert abs(float(t) / ALPHA - 1) < 1e-10
    assert tail(p + Fraction(1, 10 ** 6)) > t > tail(p - Fraction(1, 10 ** 6))


def test_cp_and_radius_against_golden_values(golden_dir):
    rows = _golden(golden_dir)
    assert len(rows) >= 20
    for n, k, p_txt, r_txt in rows:
        p = stats.cp_lower(k, n, ALPHA)
        assert p == pytest.approx(float(p_txt), rel=1e-13, abs=1e-15)
        cls, rad, p_l, n_top = stats.certify_decision([0, 5, 1], [n - k, k, 0], 64.0, n, ALPHA)
        assert n_top == k and p_l == p
        if r_txt == "abstain":
            assert cls == stats.ABSTAIN and rad == 0.0
        else:
            assert cls == 1
            # conditioning: d(radius)/radius = dp / ((p - 1/2)-ish); p carries ~1e-16 absolute error
            tol = max(1e-12, 4e-16 / abs(float(p_txt) - 0.5))
            assert rad / 64.0 == pytest.approx(float(r_txt), rel=tol)


def test_smallest_certifying_counts():
    for n, k in ((100, 66), (1000, 550), (10000, 5156), (100000, 50490)):
        assert stats.cp_lower(k, n, ALPHA) > 0.5 >= stats.cp_lower(k - 1, n, ALPHA)


def test_max_radius_brackets_from_the_papers_tables(golden_dir):
    """All N2 estimation samples in one class gives the largest radius; the
    certified-accuracy tables bracket it (non-zero column <= R_max < zero column)."""
    n_rows = 0
    for l in open(os.path.join(golden_dir, "max_radius_brackets.txt")):
        if l.startswith("#") or not l.strip():
            continue
        _, n2, sigma, last_nz, first_z = l.split()
        n2, sigma = int(n2), float(sigma)
        counts1 = [0, n2, 0]
        cls, rad, _, _ = stats.certify_decision([0, 3, 1], counts1, sigma, n2, ALPHA)
        assert cls == 1
        assert float(last_nz) <= rad < float(first_z)
        n_rows += 1
    assert n_rows == 8


def test_radius_is_sigma_times_normal_quantile():
    mp.mp.dps = 40
    for p in (0.5000001, 0.6, 0.9, 0.999, 0.99993092483300939):
        want = float(mp.sqrt(2) * mp.erfinv(2 * mp.mpf(p) - 1))
        assert stats.radius(1.0, p) == pytest.approx(want, rel=1e-12)
        assert stats.radius(128.0, p) == pytest.approx(128 * want, rel=1e-12)
    assert stats.radius(32.0, 0.5) == 0.0


def test_certify_decision_rule():
    # selection picks the lowest index among equal top counts; estimation count is read at that class
    cls, rad, p_l, k = stats.certify_decision([40, 40, 20], [900, 50, 50], 32.0, 1000, ALPHA)
    assert cls == 0 and k == 900 and rad > 0
    cls, rad, p_l, k = stats.certify_decision([10, 70, 20], [900, 50, 50], 32.0, 1000, ALPHA)
    assert cls == stats.ABSTAIN and k == 50 and rad == 0.0 and p_l < 0.5
    # bound exactly at / below one half abstains (strict inequality in Alg. 1)
    cls, _, p_l, _ = stats.certify_decision([1, 0], [50000, 50000], 32.0, 100000, ALPHA)
    assert cls == stats.ABSTAIN and p_l == pytest.approx(0.4951090429036958864, rel=1e-12)
    # radius grows with the count and with sigma
    r1 = stats.certify_decision([1, 0], [700, 300], 32.0, 1000, ALPHA)[1]
    r2 = stats.certify_decision([1, 0], [800, 200], 32.0, 1000, ALPHA)[1]
    r3 = stats.certify_decision([1, 0], [800, 200], 64.0, 1000, ALPHA)[1]
    assert 0 < r1 < r2 and r3 == pytest.approx(2 * r2, rel=1e-15)


def test_binomial_pvalue_exact():
    """min(1, 2 P[Bin(m, 1/2) >= n_A]) with exact rationals."""
    for n_a, n_b in ((60, 40), (70, 30), (550, 450), (560, 440), (12, 0), (11, 0), (10, 0), (9, 0), (5, 5), (1, 0)):
        m = n_a + n_b
        exact = min(Fraction(1), 2 * Fraction(sum(math.comb(m, j) for j in range(n_a, m + 1)), 2 ** m))
        assert stats.binom_pvalue(n_a, n_b) == pytest.approx(float(exact), rel=1e-12)
    assert stats.binom_pvalue(100, 0) == pytest.approx(2.0 ** -99, rel=1e-12)


def test_predict_decision_rule():
    cls, pv, n_a, n_b = stats.predict_decision([30, 70, 0], ALPHA)
    assert (cls, n_a, n_b) == (1, 70, 30) and pv < ALPHA
    cls, pv, n_a, n_b = stats.predict_decision([40, 60, 0], ALPHA)
    assert cls == stats.ABSTAIN and (n_a, n_b) == (60, 40) and pv == pytest.approx(0.056887933640980784, rel=1e-10)
    # ties: lowest index is the top class, the other one the runner-up
    cls, pv, n_a, n_b = stats.predict_decision([50, 50], ALPHA)
    assert cls == stats.ABSTAIN and n_a == n_b == 50 and pv == 1.0
    # single class: 11 votes are enough at alpha = 0.001, 10 are not
    assert stats.predict_decision([0, 11, 0], ALPHA)[0] == 1
    assert stats.predict_decision([0, 10, 0], ALPHA)[0] == stats.ABSTAIN
    # runner-up is the second largest count, not the second index
    assert stats.predict_decision([5, 80, 1, 14], ALPHA)[2:] == (80, 14)


def test_certified_percentage_and_accuracy_worked_example():
    """Section "Evaluation Metrics": five inputs counted by hand.  Input 1 abstains;
    input 3 certifies the wrong class; the radii of the correct ones are 0.5, 1.2, 0.1."""
    classes = [1, stats.ABSTAIN, 2, 0, 2]
    radii = [0.5, 0.0, 1.2, 0.3, 0.1]
    labels = [1, 3, 2, 1, 2]
    assert stats.certified_percentage(classes) == 4 / 5
    assert stats.certified_accuracy(classes, radii, labels, 0.0) == 3 / 4
    assert stats.certified_accuracy(classes, radii, labels, 0.2) == 2 / 4
    assert stats.certified_accuracy(classes, radii, labels, 0.5) == 2 / 4      # radius == r counts
    assert stats.certified_accuracy(classes, radii, labels, 0.51) == 1 / 4
    assert stats.certified_accuracy(classes, radii, labels, 1.3) == 0.0
    # a wrong class never counts, however large its radius
    assert stats.certified_accuracy([0], [9.0], [1], 0.0) == 0.0
    # nobody certified: CP 0 and CA defined as 0
    assert stats.certified_percentage([stats.ABSTAIN] * 3) == 0.0
    assert stats.certified_accuracy([stats.ABSTAIN] * 3, [0.0] * 3, [0, 1, 2], 0.0) == 0.0


def test_certified_accuracy_is_a_decreasing_step_function_of_the_radius():
    rng = np.random.default_rng(3)
    L = 200
    labels = rng.integers(0, 10, size=L)
    classes = np.where(rng.random(L) < 0.7, labels, rng.integers(0, 10, size=L))
    classes = np.where(rng.random(L) < 0.2, stats.ABSTAIN, classes)
    radii = np.where(classes == stats.ABSTAIN, 0.0, rng.random(L) * 100)
    cp = stats.certified_percentage(classes)
    assert cp == np.mean(classes != stats.ABSTAIN)
    grid = np.linspace(0, 110, 23)
    ca = [stats.certified_accuracy(classes, radii, labels, r) for r in grid]
    assert all(a >= b for a, b in zip(ca, ca[1:])) and ca[-1] == 0.0
    # CA(r) * CP is the share of the whole set that is certified, correct and has radius >= r
    for r, a in zip(grid, ca):
        whole = np.mean((classes != stats.ABSTAIN) & (classes == labels) & (radii >= r))
        assert a * cp == pytest.approx(whole, rel=1e-12, abs=1e-15)
