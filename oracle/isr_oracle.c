/*
 * CPU oracle for integer randomized smoothing -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, obviously-correct implementation of what the Monte-Carlo loop
 * of the paper's certification and prediction procedures computes (Alg. 1 and
 * Alg. 2): discrete-Gaussian noise on the integer pixel grid (Def. 3.3), the
 * integer-only forward pass of the quantized base classifier, and the class
 * vote tally.  It shares no code with the HIP library; only tests, the smoke
 * check and the CPU-baseline leg of the benchmark may call it.
 *
 * Conventions
 *   - images are uint8 [C][H][W]; tensors inside the network are int8
 *     [C][H][W] with a per-tensor zero-point z;
 *   - the noise law is the discrete Gaussian of Def. 3.3 on Z with location 0
 *     and scale sigma (grid units); how a uniform 64-bit word is turned into a
 *     draw is this build's specification (the paper fixes the law only):
 *     an inverse-CDF table built with integer arithmetic, indexed by a
 *     Philox4x32-10 word pair addressed by (seed, image, phase, sample, pixel);
 *   - x + delta is saturated to [0, 255] before the network sees it.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef unsigned __int128 u128;

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon et al., SC'11): counter-based generator.            */

static void mulhilo(uint32_t a, uint32_t b, uint32_t *hi, uint32_t *lo) {
    uint64_t p = (uint64_t)a * (uint64_t)b;
    *hi = (uint32_t)(p >> 32);
    *lo = (uint32_t)p;
}

void isr_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint32_t hi0, lo0, hi1, lo1;
        mulhilo(0xD2511F53u, c0, &hi0, &lo0);
        mulhilo(0xCD9E8D57u, c2, &hi1, &lo1);
        uint32_t n0 = hi1 ^ c1 ^ k0;
        uint32_t n1 = lo1;
        uint32_t n2 = hi0 ^ c3 ^ k1;
        uint32_t n3 = lo0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------------ */
/* Inverse-CDF threshold table of the discrete Gaussian N_Z(0, sigma^2),     */
/* pmf(k) proportional to exp(-k^2 / (2 sigma^2))  (Def. 3.3, location 0).   */
/*                                                                           */
/* Fixed point with 62 fractional bits.  q1 = exp(-1/D), D = 2 sigma^2, by   */
/* its alternating Taylor series; w[k] = exp(-k^2/D) by the recurrence       */
/* w[k+1] = w[k] r_k, r_{k+1} = r_k exp(-2/D), r_0 = q1.  Masses are          */
/* m[k] = w[|k|] >> 10 so that their sum W fits 64 bits; the support radius  */
/* R is the last k whose mass is not 0.  T[i] = floor(2^64 P[delta <= i-R]), */
/* which lies in [1, 2^64) for every i in [0, 2R).                           */
/* A uniform 64-bit u maps to delta = -R + #{ i in [0,2R) : T[i] <= u }.     */

#define FR 62
static uint64_t fxmul(uint64_t a, uint64_t b) { return (uint64_t)(((u128)a * (u128)b) >> FR); }

/* Returns 0 on success; writes 2R thresholds to T (needs cap >= 2R) and R.  */
int isr_oracle_noise_table(uint32_t sigma, uint64_t *T, size_t cap, uint32_t *R_out) {
    if (sigma < 1 || sigma > 1024) return -1;
    const uint64_t ONE = (uint64_t)1 << FR;
    const uint64_t D = 2ull * sigma * sigma;
    /* q1 = sum_j (-1)^j (1/D)^j / j! */
    uint64_t t = ONE, q1 = ONE;
    int negative = 1;
    for (uint64_t j = 1;; ++j) {
        t = t / (D * j);
        if (t == 0) break;
        if (negative) q1 -= t; else q1 += t;
        negative = !negative;
    }
    uint64_t g = fxmul(q1, q1);
    size_t wcap = 16384, nw = 1;
    uint64_t *w = (uint64_t *)malloc(wcap * sizeof(uint64_t));
    if (!w) return -2;
    w[0] = ONE;
    uint64_t r = q1;
    for (;;) {
        uint64_t next = fxmul(w[nw - 1], r);
        if ((next >> 10) == 0) break;
        if (nw == wcap) { free(w); return -3; }
        w[nw++] = next;
        r = fxmul(r, g);
    }
    uint32_t R = (uint32_t)(nw - 1);
    *R_out = R;
    if (cap < 2 * (size_t)R) { free(w); return -4; }
    u128 W = 0;
    for (int64_t k = -(int64_t)R; k <= (int64_t)R; ++k) W += w[k < 0 ? -k : k] >> 10;
    if (W >> 64) { free(w); return -5; }
    u128 C = 0;
    for (uint32_t i = 0; i < 2 * R; ++i) {
        int64_t k = (int64_t)i - (int64_t)R;
        C += w[k < 0 ? -k : k] >> 10;      /* C = sum of masses of all j <= k */
        T[i] = (uint64_t)((C << 64) / W);
    }
    free(w);
    return 0;
}

int32_t isr_oracle_delta(const uint64_t *T, uint32_t R, uint64_t u) {
    int32_t count = 0;
    for (uint32_t i = 0; i < 2 * R; ++i) count += (T[i] <= u);
    return count - (int32_t)R;
}

/* The 64-bit uniform word of logical pixel p = (c*H + y)*W + x:             */
/* counter (p >> 2, sample, image, (phase << 1) | half), key = seed halves;  */
/* output word (p & 3); half 0 gives the high 32 bits, half 1 the low 32.    */
uint64_t isr_oracle_uniform64(uint64_t seed, uint32_t image, uint32_t phase, uint32_t sample, uint32_t p) {
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t ctr[4] = {p >> 2, sample, image, (phase << 1) | 0u};
    uint32_t hi[4], lo[4];
    isr_oracle_philox4x32_10(ctr, key, hi);
    ctr[3] = (phase << 1) | 1u;
    isr_oracle_philox4x32_10(ctr, key, lo);
    return ((uint64_t)hi[p & 3] << 32) | lo[p & 3];
}

/* a0 = clamp(x + delta, 0, 255) - 128 for every pixel of one noisy copy.    */
void isr_oracle_noisy(const uint8_t *x, uint32_t npix, const uint64_t *T, uint32_t R, uint64_t seed,
                      uint32_t image, uint32_t phase, uint32_t sample, int8_t *a0) {
    for (uint32_t p = 0; p < npix; ++p) {
        uint64_t u = isr_oracle_uniform64(seed, image, phase, sample, p);
        int32_t v = (int32_t)x[p] + isr_oracle_delta(T, R, u);
        if (v < 0) v = 0;
        if (v > 255) v = 255;
        a0[p] = (int8_t)(v - 128);
    }
}

/* Noise stored ahead of training (training section: the noise of a batch is     */
/* sampled once and kept): draw p of tensor first + t is the table sampler on the */
/* 64-bit word of the stream with the tensor index as sample, the bank id as      */
/* image and phase 2; no image is added and nothing saturates.                    */
void isr_oracle_noise_bank(const uint64_t *T, uint32_t R, uint64_t seed, uint32_t bank, uint32_t first,
                           uint32_t count, uint32_t d, int16_t *out) {
    for (uint32_t t = 0; t < count; ++t)
        for (uint32_t p = 0; p < d; ++p)
            out[(size_t)t * d + p] = (int16_t)isr_oracle_delta(T, R, isr_oracle_uniform64(seed, bank, 2u, first + t, p));
}

/* ------------------------------------------------------------------------ */
/* Quantized network: parse the ISRM blob, run the integer forward pass.     */

enum { OP_CONV = 1, OP_ADD = 2, OP_MAXPOOL = 3, OP_GAP = 4, OP_FC = 5 };

typedef struct { int32_t C, H, W, zp; } otensor;
typedef struct {
    int32_t type;
    int32_t a, b, out;          /* tensor ids (b only for ADD) */
    int32_t k, stride, pad, relu;
    int32_t Ma, Mb, sh;         /* ADD / GAP scalars */
    const int8_t *w;            /* CONV: [Cout][Cin][k][k]; FC: [Cout][Cin] */
    const int32_t *bias, *M0, *shift;
} oop;
typedef struct {
    uint8_t *blob;
    int32_t C, H, W, classes, nt, nops;
    otensor *t;
    oop *ops;
} omodel;

static int32_t rd32(const uint8_t *p) { int32_t v; memcpy(&v, p, 4); return v; }

void isr_oracle_free(omodel *m) {
    if (!m) return;
    free(m->blob); free(m->t); free(m->ops); free(m);
}

omodel *isr_oracle_load(const void *blob, size_t bytes) {
    if (bytes < 32) return NULL;
    omodel *m = (omodel *)calloc(1, sizeof(omodel));
    m->blob = (uint8_t *)malloc(bytes);
    memcpy(m->blob, blob, bytes);
    const uint8_t *p = m->blob, *end = m->blob + bytes;
    if (rd32(p) != 0x4D525349 || rd32(p + 4) != 1) { isr_oracle_free(m); return NULL; }
    m->C = rd32(p + 8); m->H = rd32(p + 12); m->W = rd32(p + 16);
    m->classes = rd32(p + 20); m->nt = rd32(p + 24); m->nops = rd32(p + 28);
    p += 32;
    m->t = (otensor *)calloc((size_t)m->nt, sizeof(otensor));
    m->ops = (oop *)calloc((size_t)m->nops, sizeof(oop));
    for (int i = 0; i < m->nt; ++i, p += 16) {
        if (p + 16 > end) { isr_oracle_free(m); return NULL; }
        m->t[i].C = rd32(p); m->t[i].H = rd32(p + 4); m->t[i].W = rd32(p + 8); m->t[i].zp = rd32(p + 12);
    }
    for (int i = 0; i < m->nops; ++i) {
        if (p + 8 > end) { isr_oracle_free(m); return NULL; }
        oop *o = &m->ops[i];
        o->type = rd32(p);
        int32_t len = rd32(p + 4);
        const uint8_t *q = p + 8;
        if (q + len > end) { isr_oracle_free(m); return NULL; }
        switch (o->type) {
        case OP_CONV: {
            o->a = rd32(q); o->out = rd32(q + 4); o->k = rd32(q + 8); o->stride = rd32(q + 12);
            o->pad = rd32(q + 16); o->relu = rd32(q + 20);
            int32_t cin = m->t[o->a].C, cout = m->t[o->out].C;
            size_t wb = (size_t)cout * cin * o->k * o->k;
            o->w = (const int8_t *)(q + 24);
            const uint8_t *r = q + 24 + ((wb + 3) & ~(size_t)3);
            o->bias = (const int32_t *)r;
            o->M0 = o->bias + cout;
            o->shift = o->M0 + cout;
            break; }
        case OP_ADD:
            o->a = rd32(q); o->b = rd32(q + 4); o->out = rd32(q + 8); o->Ma = rd32(q + 12);
            o->Mb = rd32(q + 16); o->sh = rd32(q + 20); o->relu = rd32(q + 24);
            break;
        case OP_MAXPOOL:
            o->a = rd32(q); o->out = rd32(q + 4); o->k = rd32(q + 8); o->stride = rd32(q + 12);
            o->pad = rd32(q + 16);
            break;
        case OP_GAP:
            o->a = rd32(q); o->out = rd32(q + 4); o->Ma = rd32(q + 8); o->sh = rd32(q + 12);
            break;
        case OP_FC: {
            o->a = rd32(q); o->out = rd32(q + 4);
            otensor ti = m->t[o->a];
            size_t wb = (size_t)m->t[o->out].C * ti.C * ti.H * ti.W;
            o->w = (const int8_t *)(q + 8);
            o->bias = (const int32_t *)(q + 8 + ((wb + 3) & ~(size_t)3));
            break; }
        default: isr_oracle_free(m); return NULL;
        }
        p = q + len;
    }
    return m;
}

void isr_oracle_info(const omodel *m, int32_t *C, int32_t *H, int32_t *W, int32_t *classes, int32_t *nt) {
    *C = m->C; *H = m->H; *W = m->W; *classes = m->classes; *nt = m->nt;
}
void isr_oracle_tensor_shape(const omodel *m, int32_t id, int32_t *C, int32_t *H, int32_t *W, int32_t *zp) {
    *C = m->t[id].C; *H = m->t[id].H; *W = m->t[id].W; *zp = m->t[id].zp;
}

/* Round-half-away-from-zero division of v by 2^s (one rounding). */
int64_t isr_oracle_rha(int64_t v, int32_t s) {
    if (s == 0) return v;
    int64_t half = (int64_t)1 << (s - 1);
    return v >= 0 ? (v + half) >> s : -((-v + half) >> s);
}

static int8_t clampq(int64_t v, int32_t zp_out, int32_t relu) {
    int64_t lo = relu ? zp_out : -128;
    if (v < lo) v = lo;
    if (v > 127) v = 127;
    return (int8_t)v;
}

/* acc = bias + sum over in-bounds taps of (q - z_in) * w ; q_out = clamp(z_out + RHA(acc*M0, 31+shift)) */
static void conv_op(const omodel *m, const oop *o, const int8_t *in, int8_t *out) {
    otensor ti = m->t[o->a], to = m->t[o->out];
    int k = o->k;
    for (int oc = 0; oc < to.C; ++oc)
        for (int oy = 0; oy < to.H; ++oy)
            for (int ox = 0; ox < to.W; ++ox) {
                int32_t acc = o->bias[oc];
                for (int ic = 0; ic < ti.C; ++ic)
                    for (int ky = 0; ky < k; ++ky) {
                        int iy = oy * o->stride - o->pad + ky;
                        if (iy < 0 || iy >= ti.H) continue;
                        for (int kx = 0; kx < k; ++kx) {
                            int ix = ox * o->stride - o->pad + kx;
                            if (ix < 0 || ix >= ti.W) continue;
                            int32_t q = in[((size_t)ic * ti.H + iy) * ti.W + ix];
                            int32_t wv = o->w[(((size_t)oc * ti.C + ic) * k + ky) * k + kx];
                            acc += (q - ti.zp) * wv;
                        }
                    }
                int64_t r = isr_oracle_rha((int64_t)acc * (int64_t)o->M0[oc], 31 + o->shift[oc]);
                out[((size_t)oc * to.H + oy) * to.W + ox] = clampq(to.zp + r, to.zp, o->relu);
            }
}

static void add_op(const omodel *m, const oop *o, const int8_t *a, const int8_t *b, int8_t *out) {
    otensor ta = m->t[o->a], tb = m->t[o->b], to = m->t[o->out];
    size_t n = (size_t)to.C * to.H * to.W;
    for (size_t i = 0; i < n; ++i) {
        int64_t v = (int64_t)(a[i] - ta.zp) * o->Ma + (int64_t)(b[i] - tb.zp) * o->Mb;
        out[i] = clampq(to.zp + isr_oracle_rha(v, o->sh), to.zp, o->relu);
    }
}

static void maxpool_op(const omodel *m, const oop *o, const int8_t *in, int8_t *out) {
    otensor ti = m->t[o->a], to = m->t[o->out];
    for (int c = 0; c < to.C; ++c)
        for (int oy = 0; oy < to.H; ++oy)
            for (int ox = 0; ox < to.W; ++ox) {
                int best = -129;
                for (int ky = 0; ky < o->k; ++ky)
                    for (int kx = 0; kx < o->k; ++kx) {
                        int iy = oy * o->stride - o->pad + ky, ix = ox * o->stride - o->pad + kx;
                        if (iy < 0 || iy >= ti.H || ix < 0 || ix >= ti.W) continue;
                        int q = in[((size_t)c * ti.H + iy) * ti.W + ix];
                        if (q > best) best = q;
                    }
                out[((size_t)c * to.H + oy) * to.W + ox] = (int8_t)best;
            }
}

static void gap_op(const omodel *m, const oop *o, const int8_t *in, int8_t *out) {
    otensor ti = m->t[o->a], to = m->t[o->out];
    for (int c = 0; c < ti.C; ++c) {
        int32_t S = 0;
        for (int i = 0; i < ti.H * ti.W; ++i) S += in[(size_t)c * ti.H * ti.W + i] - ti.zp;
        int64_t r = isr_oracle_rha((int64_t)S * (int64_t)o->Ma, 31 + o->sh);
        out[c] = clampq(to.zp + r, to.zp, 0);
    }
}

static void fc_op(const omodel *m, const oop *o, const int8_t *in, int32_t *logits) {
    otensor ti = m->t[o->a], to = m->t[o->out];
    int cin = ti.C * ti.H * ti.W;
    for (int oc = 0; oc < to.C; ++oc) {
        int32_t acc = o->bias[oc];
        for (int i = 0; i < cin; ++i) acc += (in[i] - ti.zp) * (int32_t)o->w[(size_t)oc * cin + i];
        logits[oc] = acc;
    }
}

size_t isr_oracle_tensor_offset(const omodel *m, int32_t id) {
    size_t off = 0;
    for (int i = 0; i < id; ++i) off += (size_t)m->t[i].C * m->t[i].H * m->t[i].W;
    return off;
}

/* Forward pass of one noisy copy a0 (int8 [C][H][W]).  `acts` holds every
 * int8 tensor back to back (offsets from isr_oracle_tensor_offset; the logits
 * tensor's slot is left unused); logits gets `classes` int32 values.         */
int isr_oracle_forward(const omodel *m, const int8_t *a0, int8_t *acts, int32_t *logits) {
    size_t *off = (size_t *)malloc((size_t)m->nt * sizeof(size_t));
    for (int i = 0; i < m->nt; ++i) off[i] = isr_oracle_tensor_offset(m, i);
    memcpy(acts, a0, (size_t)m->C * m->H * m->W);
    for (int i = 0; i < m->nops; ++i) {
        const oop *o = &m->ops[i];
        switch (o->type) {
        case OP_CONV: conv_op(m, o, acts + off[o->a], acts + off[o->out]); break;
        case OP_ADD: add_op(m, o, acts + off[o->a], acts + off[o->b], acts + off[o->out]); break;
        case OP_MAXPOOL: maxpool_op(m, o, acts + off[o->a], acts + off[o->out]); break;
        case OP_GAP: gap_op(m, o, acts + off[o->a], acts + off[o->out]); break;
        case OP_FC: fc_op(m, o, acts + off[o->a], logits); break;
        }
    }
    free(off);
    return 0;
}

/* Lowest index among the maxima. */
int32_t isr_oracle_argmax(const int32_t *v, int32_t n) {
    int32_t best = 0;
    for (int32_t i = 1; i < n; ++i) if (v[i] > v[best]) best = i;
    return best;
}

/* Monte-Carlo loop over sample indices [begin, begin+count) of one phase:
 * noisy copy -> forward -> argmax -> vote.  Any of logits (count*classes),
 * argmax (count), counts (classes, accumulated into) may be NULL.  Samples
 * are independent, so the loop is split over `threads` OpenMP threads.       */
int isr_oracle_mc(const omodel *m, const uint8_t *x, uint32_t sigma, uint64_t seed, uint32_t image,
                  uint32_t phase, uint32_t begin, uint32_t count, int32_t *logits, int32_t *argmax,
                  uint32_t *counts, int threads) {
    uint32_t R = 0;
    uint64_t *T = (uint64_t *)malloc(2 * 16384 * sizeof(uint64_t));
    if (isr_oracle_noise_table(sigma, T, 2 * 16384, &R) != 0) { free(T); return -1; }
    uint32_t npix = (uint32_t)(m->C * m->H * m->W);
    size_t total = isr_oracle_tensor_offset(m, m->nt);
    int32_t *am = (int32_t *)malloc((size_t)count * sizeof(int32_t));
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
    {
        int8_t *a0 = (int8_t *)malloc(npix);
        int8_t *acts = (int8_t *)malloc(total);
        int32_t *lg = (int32_t *)malloc((size_t)m->classes * sizeof(int32_t));
#pragma omp for schedule(dynamic, 1)
        for (uint32_t s = 0; s < count; ++s) {
            isr_oracle_noisy(x, npix, T, R, seed, image, phase, begin + s, a0);
            isr_oracle_forward(m, a0, acts, lg);
            am[s] = isr_oracle_argmax(lg, m->classes);
            if (logits) memcpy(logits + (size_t)s * m->classes, lg, (size_t)m->classes * sizeof(int32_t));
        }
        free(a0); free(acts); free(lg);
    }
    for (uint32_t s = 0; s < count; ++s) {
        if (argmax) argmax[s] = am[s];
        if (counts) counts[am[s]] += 1;
    }
    free(am); free(T);
    return 0;
}
