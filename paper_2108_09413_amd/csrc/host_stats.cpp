// Host-side decisions of the certification procedure (Alg. 1) and the
// prediction procedure (Alg. 2): Clopper-Pearson lower bound, standard normal
// quantile, two-sided binomial test.  float64 results computed in long double.
#include <cmath>
#include <cstdint>

#include "isr.h"

namespace {

typedef long double ld;

// Continued fraction of the regularised incomplete beta function (modified
// Lentz evaluation); valid and fast for x < (a+1)/(a+b+2).
ld beta_cf(ld a, ld b, ld x) {
    const ld tiny = 1e-4000L, eps = 1e-20L;
    ld c = 1.0L, d = 1.0L - (a + b) * x / (a + 1.0L);
    if (fabsl(d) < tiny) d = tiny;
    d = 1.0L / d;
    ld h = d;
    for (int m = 1; m < 200000; ++m) {
        ld m2 = 2.0L * m;
        ld num = m * (b - m) * x / ((a + m2 - 1.0L) * (a + m2));
        d = 1.0L + num * d; if (fabsl(d) < tiny) d = tiny;
        c = 1.0L + num / c; if (fabsl(c) < tiny) c = tiny;
        d = 1.0L / d;
        h *= d * c;
        num = -(a + m) * (a + b + m) * x / ((a + m2) * (a + m2 + 1.0L));
        d = 1.0L + num * d; if (fabsl(d) < tiny) d = tiny;
        c = 1.0L + num / c; if (fabsl(c) < tiny) c = tiny;
        d = 1.0L / d;
        ld del = d * c;
        h *= del;
        if (fabsl(del - 1.0L) < eps) break;
    }
    return h;
}

ld log_beta_fn(ld a, ld b) { return lgammal(a) + lgammal(b) - lgammal(a + b); }

// I_x(a, b), a, b > 0, 0 <= x <= 1.
ld inc_beta(ld a, ld b, ld x) {
    if (x <= 0.0L) return 0.0L;
    if (x >= 1.0L) return 1.0L;
    ld lpre = a * logl(x) + b * log1pl(-x) - log_beta_fn(a, b);
    if (x < (a + 1.0L) / (a + b + 2.0L)) return expl(lpre) * beta_cf(a, b, x) / a;
    return 1.0L - expl(lpre) * beta_cf(b, a, 1.0L - x) / b;
}

// Density of Beta(a, b) at x = d/dx I_x(a, b).
ld beta_pdf(ld a, ld b, ld x) {
    return expl((a - 1.0L) * logl(x) + (b - 1.0L) * log1pl(-x) - log_beta_fn(a, b));
}

// Upper tail of the standard normal.
ld norm_sf(ld x) { return 0.5L * erfcl(x * 0.70710678118654752440084436210484903928L); }

}  // namespace

extern "C" int isr_cp_lower(uint32_t k, uint32_t n, double alpha, double *p_lower) {
    if (!p_lower || n == 0 || k > n || !(alpha > 0.0 && alpha < 1.0)) return ISR_ERR_ARG;
    if (k == 0) { *p_lower = 0.0; return ISR_OK; }
    if (k == n) { *p_lower = (double)expl(logl((ld)alpha) / (ld)n); return ISR_OK; }
    // Root in p of P[Bin(n, p) >= k] = I_p(k, n-k+1) = alpha: safeguarded Newton.
    const ld a = k, b = (ld)n - k + 1.0L, target = alpha;
    ld lo = 0.0L, hi = 1.0L;
    ld ph = a / (a + b);
    ld p = ph - 3.0L * sqrtl(ph * (1.0L - ph) / (ld)n);
    if (!(p > 0.0L)) p = ph * 0.5L;
    for (int it = 0; it < 300; ++it) {
        ld f = inc_beta(a, b, p) - target;
        if (f > 0.0L) hi = p; else lo = p;
        ld dens = beta_pdf(a, b, p);
        ld next = (dens > 0.0L && std::isfinite((double)(f / dens))) ? p - f / dens : 0.5L * (lo + hi);
        if (!(next > lo && next < hi)) next = 0.5L * (lo + hi);
        ld step = fabsl(next - p);
        p = next;
        if (step <= 1e-19L * p || hi - lo <= 1e-19L * hi) break;
    }
    *p_lower = (double)p;
    return ISR_OK;
}

extern "C" int isr_normal_quantile(double p, double *z) {
    if (!z || !(p > 0.0 && p < 1.0)) return ISR_ERR_ARG;
    if (p == 0.5) { *z = 0.0; return ISR_OK; }
    // Solve the upper-tail equation on the side where the tail is <= 1/2.
    const bool upper = p > 0.5;
    const ld q = upper ? (ld)1.0 - (ld)p : (ld)p;  // exact in long double
    const ld lq = logl(q);
    ld lo = 0.0L, hi = 40.0L;
    ld x = q > 0.1L ? (0.5L - q) * 2.5066282746310005024L : sqrtl(-2.0L * lq);
    if (x >= hi) x = 0.5L * hi;
    for (int it = 0; it < 200; ++it) {
        ld sf = norm_sf(x);
        ld g = logl(sf) - lq;              // decreasing in x
        if (g > 0.0L) lo = x; else hi = x;
        ld dens = 0.39894228040143267793994605993438L * expl(-0.5L * x * x);
        ld next = x + g * sf / dens;       // Newton on log tail
        if (!(next > lo && next < hi)) next = 0.5L * (lo + hi);
        ld step = fabsl(next - x);
        x = next;
        if (step <= 1e-19L * fabsl(x) || hi - lo <= 1e-19L * hi) break;
    }
    *z = (double)(upper ? x : -x);
    return ISR_OK;
}

extern "C" int isr_binom_pvalue(uint32_t n_a, uint32_t n_b, double *pvalue) {
    if (!pvalue) return ISR_ERR_ARG;
    if (n_a == 0) { *pvalue = 1.0; return ISR_OK; }
    // P[Bin(m, 1/2) >= n_a] = I_{1/2}(n_a, m - n_a + 1), m = n_a + n_b
    ld tail = inc_beta((ld)n_a, (ld)n_b + 1.0L, 0.5L);
    ld pv = 2.0L * tail;
    *pvalue = (double)(pv > 1.0L ? 1.0L : pv);
    return ISR_OK;
}

static uint32_t lowest_argmax(const uint32_t *c, uint32_t n) {
    uint32_t best = 0;
    for (uint32_t i = 1; i < n; ++i) if (c[i] > c[best]) best = i;
    return best;
}

extern "C" int isr_decide_certify(const uint32_t *counts0, const uint32_t *counts1, uint32_t classes,
                                  double sigma, uint32_t n, double alpha, isr_result *out) {
    if (!counts0 || !counts1 || !out || classes == 0 || !(sigma > 0.0)) return ISR_ERR_ARG;
    uint32_t ca = lowest_argmax(counts0, classes);
    uint32_t k = counts1[ca];
    double pl = 0.0;
    int rc = isr_cp_lower(k, n, alpha, &pl);
    if (rc != ISR_OK) return rc;
    out->n_top = k;
    out->n_second = 0;
    out->p_lower = pl;
    out->radius_int = 0;
    out->radius_sq_int = 0;
    if (pl > 0.5) {
        double z = 0.0;
        rc = isr_normal_quantile(pl, &z);
        if (rc != ISR_OK) return rc;
        out->cls = (int32_t)ca;
        out->radius = sigma * z;
        // integer-only tail (Thm 3.2, proof steps 2-3): quantile of the discrete law by table lookup
        if (sigma >= 1.0 && sigma <= 1024.0 && sigma == std::floor(sigma)) {
            rc = isr_discrete_quantile((uint32_t)sigma, pl, &out->radius_int, &out->radius_sq_int);
            if (rc != ISR_OK) return rc;
        }
    } else {
        out->cls = ISR_ABSTAIN;
        out->radius = 0.0;
    }
    return ISR_OK;
}

extern "C" int isr_decide_predict(const uint32_t *counts, uint32_t classes, double alpha, isr_result *out) {
    if (!counts || !out || classes == 0 || !(alpha > 0.0 && alpha < 1.0)) return ISR_ERR_ARG;
    uint32_t ca = lowest_argmax(counts, classes);
    uint32_t nb = 0;
    for (uint32_t i = 0; i < classes; ++i) if (i != ca && counts[i] > nb) nb = counts[i];
    double pv = 1.0;
    int rc = isr_binom_pvalue(counts[ca], nb, &pv);
    if (rc != ISR_OK) return rc;
    out->radius_int = 0;
    out->radius_sq_int = 0;
    out->n_top = counts[ca];
    out->n_second = nb;
    out->p_lower = pv;
    out->radius = 0.0;
    out->cls = pv <= alpha ? (int32_t)ca : ISR_ABSTAIN;
    return ISR_OK;
}

extern "C" int isr_certified_metrics(const isr_result *results, const int32_t *labels, uint32_t count, const double *radii,
                                     uint32_t n_radii, double *cp_out, double *ca_out) {
    if (!results || count == 0 || (n_radii && (!radii || !ca_out || !labels))) return ISR_ERR_ARG;
    uint32_t certified = 0;
    for (uint32_t i = 0; i < count; ++i) certified += results[i].cls != ISR_ABSTAIN;
    if (cp_out) *cp_out = (double)certified / (double)count;
    for (uint32_t j = 0; j < n_radii; ++j) {
        uint32_t hit = 0;
        for (uint32_t i = 0; i < count; ++i)
            hit += results[i].cls != ISR_ABSTAIN && results[i].cls == labels[i] && results[i].radius >= radii[j];
        ca_out[j] = certified ? (double)hit / (double)certified : 0.0;
    }
    return ISR_OK;
}
