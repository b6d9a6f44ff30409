"""Writes cp_radius_values.txt from first principles with 50-digit mpmath.

p_lower is the root in p of  sum_{j>=k} C(n,j) p^j (1-p)^(n-j) = alpha  (the
definition of the one-sided Clopper-Pearson bound used by Alg. 1), found by
Newton iteration on the tail summed term by term; the radius factor is the
standard normal quantile of p_lower.  Uses neither scipy nor the oracle."""
import os

import mpmath as mp

mp.mp.dps = 60
ALPHA = mp.mpf("0.001")
CASES = [(100, 100), (1000, 1000), (10000, 10000), (100000, 100000),
         (100, 66), (100, 65), (1000, 550), (1000, 549), (10000, 5156), (10000, 5155),
         (100000, 50490), (100000, 50489), (100000, 50500), (100000, 50000),
         (1000, 999), (1000, 990), (1000, 900), (1000, 600), (1000, 551),
         (10000, 9900), (100000, 99000), (100000, 99999), (100000, 1), (100000, 73211)]


def log_pmf(n, j, p):
    return (mp.loggamma(n + 1) - mp.loggamma(j + 1) - mp.loggamma(n - j + 1)
            + j * mp.log(p) + (n - j) * mp.log(1 - p))


def tail(n, k, p):
    """P[Bin(n, p) >= k], summing pmf terms upward from k by their ratio."""
    term = mp.e ** log_pmf(n, k, p)
    total, j, odds = term, k, p / (1 - p)
    while j < n:
        term = term * (n - j) / (j + 1) * odds
        j += 1
        total += term
        if term < total * mp.mpf(10) ** -60:
            break
    return total


def cp_lower(n, k):
    if k == n:
        return ALPHA ** (mp.mpf(1) / n)
    # start at the normal approximation of the root (z = 3.09 for alpha = 0.001)
    ph = mp.mpf(k) / n
    p = ph - mp.mpf("3.09") * mp.sqrt(ph * (1 - ph) / n)
    p = max(p, ph / 1000)
    for _ in range(60):
        f = tail(n, k, p) - ALPHA
        dens = k * mp.e ** log_pmf(n, k, p) / p      # d/dp P[Bin(n,p) >= k]
        step = f / dens
        while not (0 < p - step < 1):
            step /= 2
        p = p - step
        if abs(step) < mp.mpf(10) ** -40:
            break
    assert abs(tail(n, k, p) / ALPHA - 1) < mp.mpf(10) ** -35
    return p


def main():
    here = os.path.dirname(os.path.abspath(__file__))
    path = os.path.join(here, "cp_radius_values.txt")
    head = [l for l in open(path) if l.startswith("#")]
    with open(path, "w") as f:
        f.writelines(head)
        for n, k in CASES:
            p = cp_lower(n, k)
            r = "abstain" if p <= mp.mpf("0.5") else mp.nstr(mp.sqrt(2) * mp.erfinv(2 * p - 1), 20)
            f.write(f"{n} {k} {mp.nstr(p, 20)} {r}\n")


if __name__ == "__main__":
    main()
