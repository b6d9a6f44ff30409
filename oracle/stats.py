"""Host-side statistics of the oracle (float64) -- TEST INFRASTRUCTURE ONLY.

The decision rules of the certification procedure (Alg. 1) and the prediction
procedure (Alg. 2), written with library routines as the individual steps.
"""
from __future__ import annotations

from scipy import stats as _st

ABSTAIN = -1


def cp_lower(k: int, n: int, alpha: float) -> float:
    """One-sided (1 - alpha) Clopper-Pearson lower confidence bound on a
    binomial proportion after k successes in n trials (Alg. 1, the step that
    defines the lower bound p_A; the exact interval of the cited smoothing
    work): the p at which P[Bin(n, p) >= k] = alpha, i.e. the alpha-quantile of
    Beta(k, n - k + 1); 0 when k = 0."""
    if k == 0:
        return 0.0
    return float(_st.beta.ppf(alpha, k, n - k + 1))


def radius(sigma: float, p_lower: float) -> float:
    """Certified l2 radius sigma * Phi^{-1}(p_A) (Alg. 1, return step), Phi the
    standard normal cdf."""
    return float(sigma * _st.norm.ppf(p_lower))


def discrete_quantile(sigma: int, p_lower: float) -> int:
    """Integer-only tail of the certification (Thm 3.2, proof steps 2 and 3): the inverse
    cdf of the one-dimensional discrete Gaussian N_Z(0, sigma^2) (Def. 3.3) by lookup in
    its precomputed cdf table -- the largest lattice point t, in input grid units, with
    P[delta <= t] <= p_lower.  With Phi^-1 of the discrete law in place of the normal
    one the radius sigma * Phi^-1(p) of Alg. 1 is t itself and the squared radius
    t * t stays on the lattice.  The cdf is the 64-bit fixed-point table of the sampler:
    T[i] = floor(2^64 P[delta <= i - R]); p_lower enters as floor(2^64 p_lower), exact
    for a float64 below 1.  Returns -R - 1 when even the first table entry exceeds p."""
    from fractions import Fraction

    from . import noise_table
    T, R = noise_table(int(sigma))
    if not 0.0 <= p_lower <= 1.0:
        raise ValueError("p_lower outside [0, 1]")
    u = min(int(Fraction(p_lower) * (1 << 64)), (1 << 64) - 1)
    below = sum(1 for t in T if int(t) <= u)
    return -R - 1 + below


def radius_squared_int(sigma: int, p_lower: float) -> int:
    """Squared certified radius in squared grid units, integers only: 0 unless the
    discrete quantile is positive (Thm 3.2, proof step 3)."""
    t = discrete_quantile(sigma, p_lower)
    return t * t if t > 0 else 0


def lowest_argmax(counts) -> int:
    best = 0
    for i in range(1, len(counts)):
        if counts[i] > counts[best]:
            best = i
    return best


def certify_decision(counts0, counts1, sigma: float, n: int, alpha: float):
    """Alg. 1 after the two Monte-Carlo loops: returns (class, radius, p_lower,
    n_top); class is ABSTAIN and radius 0.0 when the bound is not above 1/2."""
    c_a = lowest_argmax(counts0)
    k = int(counts1[c_a])
    p_l = cp_lower(k, n, alpha)
    if p_l > 0.5:
        return c_a, radius(sigma, p_l), p_l, k
    return ABSTAIN, 0.0, p_l, k


def certify_decision_integer(counts0, counts1, sigma: int, n: int, alpha: float):
    """Alg. 1 with the integer-only tail of Thm 3.2 (proof steps 2 and 3): the class and the
    bound as in certify_decision, then the radius read off the discrete Gaussian's own cdf
    table instead of sigma * Phi^-1 -- returns (class, t, t * t or 0); (ABSTAIN, 0, 0) when
    the bound is not above 1/2.  t may be <= 0 for a bound barely above 1/2: the class is
    returned with squared radius 0."""
    c_a = lowest_argmax(counts0)
    p_l = cp_lower(int(counts1[c_a]), n, alpha)
    if not p_l > 0.5:
        return ABSTAIN, 0, 0
    return c_a, discrete_quantile(sigma, p_l), radius_squared_int(sigma, p_l)


def binom_pvalue(n_a: int, n_b: int) -> float:
    """Two-sided p-value of the hypothesis that n_a successes out of
    n_a + n_b trials come from a fair coin (Alg. 2, the binomial test):
    min(1, 2 * P[Bin(n_a + n_b, 1/2) >= n_a]) for n_a >= n_b."""
    m = n_a + n_b
    return float(min(1.0, 2.0 * _st.binom.sf(n_a - 1, m, 0.5)))


def predict_decision(counts, alpha: float):
    """Alg. 2 after the Monte-Carlo loop: (class or ABSTAIN, p-value, n_A, n_B).
    The top two classes are taken with lowest index winning ties; the class is
    returned when the p-value is at most alpha."""
    c_a = lowest_argmax(counts)
    rest = [(-int(c), i) for i, c in enumerate(counts) if i != c_a]
    n_b = -min(rest)[0] if rest else 0
    n_a = int(counts[c_a])
    pv = binom_pvalue(n_a, n_b)
    return (c_a if pv <= alpha else ABSTAIN), pv, n_a, n_b


def certified_percentage(classes) -> float:
    """Certified percentage CP (section "Evaluation Metrics", first formula): the share
    of the L inputs whose certification did not abstain.  classes: the returned class
    per input, ABSTAIN where the procedure abstained."""
    classes = list(classes)
    return sum(1 for c in classes if c != ABSTAIN) / len(classes)


def certified_accuracy(classes, radii, labels, r: float) -> float:
    """Certified accuracy CA at radius r (section "Evaluation Metrics", second formula):
    among the inputs that did not abstain, the share with the correct class and a
    certified radius of at least r.  The denominator is the number of non-abstaining
    inputs, as the formula prints it (the sentence before it says "fraction of the test
    set"; CA * CP is that fraction); 0 when every input abstained."""
    classes, radii, labels = list(classes), list(radii), list(labels)
    certified = [i for i, c in enumerate(classes) if c != ABSTAIN]
    if not certified:
        return 0.0
    good = [i for i in certified if classes[i] == labels[i] and radii[i] >= r]
    return len(good) / len(certified)
