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
#include <math.h>
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

/* Output extent of a sliding window: floor((in + 2 pad - k) / stride) + 1. */
static int32_t window_out(int32_t in, int32_t k, int32_t stride, int32_t pad) { return (in + 2 * pad - k) / stride + 1; }

/* Structural checks of one op against the tensor table; payload = the op's `len` bytes.
 * Returns 1 when the op is well-formed (ids in range, inputs produced earlier, output not
 * yet produced, shapes consistent, payload exactly as long as its fields and arrays). */
static int op_is_sound(const omodel *m, const oop *o, const char *made, size_t len) {
    const int32_t nt = m->nt;
#define ID_OK(id) ((id) >= 0 && (id) < nt)
    switch (o->type) {
    case OP_CONV: {
        if (!ID_OK(o->a) || !ID_OK(o->out) || !made[o->a] || made[o->out]) return 0;
        const otensor *ti = &m->t[o->a], *to = &m->t[o->out];
        if (o->k < 1 || o->k > 15 || o->stride < 1 || o->stride > 8 || o->pad < 0 || o->pad >= o->k) return 0;
        if (o->relu != 0 && o->relu != 1) return 0;
        if (ti->H + 2 * o->pad < o->k || ti->W + 2 * o->pad < o->k) return 0;
        if (to->H != window_out(ti->H, o->k, o->stride, o->pad) || to->W != window_out(ti->W, o->k, o->stride, o->pad)) return 0;
        size_t wb = (size_t)to->C * ti->C * o->k * o->k;
        if (len != 24 + ((wb + 3) & ~(size_t)3) + 3 * (size_t)to->C * 4) return 0;
        int64_t worst = (int64_t)ti->C * o->k * o->k * 255 * 127;   /* largest |sum of products| of int8 operands */
        for (int32_t c = 0; c < to->C; ++c) {
            if (o->M0[c] < (1 << 30) || o->shift[c] < 0 || o->shift[c] > 31) return 0;
            int64_t ab = o->bias[c] < 0 ? -(int64_t)o->bias[c] : o->bias[c];
            if (worst + ab >= ((int64_t)1 << 31)) return 0;           /* the int32 accumulator must not overflow */
        }
        for (size_t i = 0; i < wb; ++i)
            if (o->w[i] == -128) return 0;
        return 1; }
    case OP_ADD: {
        if (len != 28 || !ID_OK(o->a) || !ID_OK(o->b) || !ID_OK(o->out) || !made[o->a] || !made[o->b] || made[o->out]) return 0;
        const otensor *ta = &m->t[o->a], *tb = &m->t[o->b], *to = &m->t[o->out];
        if (ta->C != tb->C || ta->H != tb->H || ta->W != tb->W || ta->C != to->C || ta->H != to->H || ta->W != to->W) return 0;
        return o->sh >= 0 && o->sh <= 40 && (o->relu == 0 || o->relu == 1); }
    case OP_MAXPOOL: {
        if (len != 20 || !ID_OK(o->a) || !ID_OK(o->out) || !made[o->a] || made[o->out]) return 0;
        const otensor *ti = &m->t[o->a], *to = &m->t[o->out];
        if (o->k < 1 || o->k > 15 || o->stride < 1 || o->stride > 8 || o->pad < 0 || o->pad >= o->k) return 0;
        if (ti->H + 2 * o->pad < o->k || ti->W + 2 * o->pad < o->k || to->C != ti->C || to->zp != ti->zp) return 0;
        return to->H == window_out(ti->H, o->k, o->stride, o->pad) && to->W == window_out(ti->W, o->k, o->stride, o->pad); }
    case OP_GAP: {
        if (len != 16 || !ID_OK(o->a) || !ID_OK(o->out) || !made[o->a] || made[o->out]) return 0;
        const otensor *ti = &m->t[o->a], *to = &m->t[o->out];
        if ((int64_t)ti->H * ti->W * 255 >= ((int64_t)1 << 31)) return 0;   /* the int32 sum must not overflow */
        return to->C == ti->C && to->H == 1 && to->W == 1 && o->Ma >= (1 << 30) && o->sh >= 0 && o->sh <= 31; }
    case OP_FC: {
        if (!ID_OK(o->a) || !ID_OK(o->out) || !made[o->a] || made[o->out]) return 0;
        const otensor *ti = &m->t[o->a], *to = &m->t[o->out];
        if (to->C != m->classes || to->H != 1 || to->W != 1) return 0;
        size_t wb = (size_t)to->C * ti->C * ti->H * ti->W;
        if (len != 8 + ((wb + 3) & ~(size_t)3) + (size_t)to->C * 4) return 0;
        int64_t worst = (int64_t)ti->C * ti->H * ti->W * 255 * 127;
        for (int32_t c = 0; c < to->C; ++c) {
            int64_t ab = o->bias[c] < 0 ? -(int64_t)o->bias[c] : o->bias[c];
            if (worst + ab >= ((int64_t)1 << 31)) return 0;
        }
        for (size_t i = 0; i < wb; ++i)
            if (o->w[i] == -128) return 0;
        return 1; }
    default: return 0;
    }
#undef ID_OK
}

/* Parses a blob; NULL when it is truncated, inconsistent or outside the format's ranges
 * (no field of a rejected blob is ever used as an index or a size). */
omodel *isr_oracle_load(const void *blob, size_t bytes) {
    if (!blob || bytes < 32) return NULL;
    omodel *m = (omodel *)calloc(1, sizeof(omodel));
    char *made = NULL;   /* per tensor: produced by an earlier op (or the input) */
    if (!m) return NULL;
    m->blob = (uint8_t *)malloc(bytes);
    if (!m->blob) { free(m); return NULL; }
    memcpy(m->blob, blob, bytes);
    const uint8_t *p = m->blob, *end = m->blob + bytes;
    if (rd32(p) != 0x4D525349 || rd32(p + 4) != 1) goto reject;
    m->C = rd32(p + 8); m->H = rd32(p + 12); m->W = rd32(p + 16);
    m->classes = rd32(p + 20); m->nt = rd32(p + 24); m->nops = rd32(p + 28);
    p += 32;
    if (m->nt < 2 || m->nt > 100000 || m->nops < 1 || m->nops > 100000 || m->classes < 1) goto reject;
    if ((size_t)(end - p) < (size_t)m->nt * 16) goto reject;
    m->t = (otensor *)calloc((size_t)m->nt, sizeof(otensor));
    m->ops = (oop *)calloc((size_t)m->nops, sizeof(oop));
    made = (char *)calloc((size_t)m->nt, 1);
    if (!m->t || !m->ops || !made) goto reject;
    for (int i = 0; i < m->nt; ++i, p += 16) {
        otensor *t = &m->t[i];
        t->C = rd32(p); t->H = rd32(p + 4); t->W = rd32(p + 8); t->zp = rd32(p + 12);
        if (t->C < 1 || t->C > 65536 || t->H < 1 || t->H > 4096 || t->W < 1 || t->W > 4096 || t->zp < -128 || t->zp > 127) goto reject;
    }
    if (m->t[0].C != m->C || m->t[0].H != m->H || m->t[0].W != m->W) goto reject;
    made[0] = 1;
    for (int i = 0; i < m->nops; ++i) {
        if ((size_t)(end - p) < 8) goto reject;
        oop *o = &m->ops[i];
        o->type = rd32(p);
        int32_t len = rd32(p + 4);
        const uint8_t *q = p + 8;
        if (len < 0 || (len & 3) || (size_t)(end - q) < (size_t)len) goto reject;
        if (i > 0 && m->ops[i - 1].type == OP_FC) goto reject;   /* the logits end the network */
        /* fixed fields first (their count is checked against len), arrays only after the ids are known good */
        switch (o->type) {
        case OP_CONV: {
            if (len < 24) goto reject;
            o->a = rd32(q); o->out = rd32(q + 4); o->k = rd32(q + 8); o->stride = rd32(q + 12);
            o->pad = rd32(q + 16); o->relu = rd32(q + 20);
            if (o->a < 0 || o->a >= m->nt || o->out < 0 || o->out >= m->nt || o->k < 1 || o->k > 15) goto reject;
            int32_t cin = m->t[o->a].C, cout = m->t[o->out].C;
            size_t wb = (size_t)cout * cin * o->k * o->k;
            if ((size_t)len != 24 + ((wb + 3) & ~(size_t)3) + 3 * (size_t)cout * 4) goto reject;
            o->w = (const int8_t *)(q + 24);
            const uint8_t *r = q + 24 + ((wb + 3) & ~(size_t)3);
            o->bias = (const int32_t *)r;
            o->M0 = o->bias + cout;
            o->shift = o->M0 + cout;
            break; }
        case OP_ADD:
            if (len != 28) goto reject;
            o->a = rd32(q); o->b = rd32(q + 4); o->out = rd32(q + 8); o->Ma = rd32(q + 12);
            o->Mb = rd32(q + 16); o->sh = rd32(q + 20); o->relu = rd32(q + 24);
            break;
        case OP_MAXPOOL:
            if (len != 20) goto reject;
            o->a = rd32(q); o->out = rd32(q + 4); o->k = rd32(q + 8); o->stride = rd32(q + 12);
            o->pad = rd32(q + 16);
            break;
        case OP_GAP:
            if (len != 16) goto reject;
            o->a = rd32(q); o->out = rd32(q + 4); o->Ma = rd32(q + 8); o->sh = rd32(q + 12);
            break;
        case OP_FC: {
            if (len < 8) goto reject;
            o->a = rd32(q); o->out = rd32(q + 4);
            if (o->a < 0 || o->a >= m->nt || o->out < 0 || o->out >= m->nt) goto reject;
            otensor ti = m->t[o->a];
            size_t wb = (size_t)m->t[o->out].C * ti.C * ti.H * ti.W;
            if ((size_t)len != 8 + ((wb + 3) & ~(size_t)3) + (size_t)m->t[o->out].C * 4) goto reject;
            o->w = (const int8_t *)(q + 8);
            o->bias = (const int32_t *)(q + 8 + ((wb + 3) & ~(size_t)3));
            break; }
        default: goto reject;
        }
        if (!op_is_sound(m, o, made, (size_t)len)) goto reject;
        made[o->out] = 1;
        p = q + len;
    }
    if (p != end || m->ops[m->nops - 1].type != OP_FC) goto reject;
    free(made);
    return m;
reject:
    free(made);
    isr_oracle_free(m);
    return NULL;
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

/* ------------------------------------------------------------------------ */
/* The two floating-point comparison systems of the paper's evaluation       */
/* (section "Experiments": FloatRS-quant and FloatRS-fp): standard           */
/* randomized smoothing with continuous Gaussian noise N(0, sigma^2 I),      */
/*   FloatRS-quant: the noisy image is rounded back onto the 8-bit pixel     */
/*                  grid and classified by the quantized network;            */
/*   FloatRS-fp:    the noisy image is classified by the float network.      */
/* The paper fixes the law only.  How a counter turns into a float32 normal  */
/* draw is this build's specification, written so that every step is an      */
/* IEEE-754 binary32 operation (+, -, *, /, sqrt, each rounded once, none    */
/* contracted) and therefore has one result on every conforming machine:     */
/*   Philox4x32-10, counter (p >> 2, sample, image, 8 + phase), key = seed;  */
/*   words (w0, w1) give the draws of elements p&3 = 0, 1, words (w2, w3)    */
/*   those of elements 2, 3 by the Box-Muller transform                      */
/*   z_a = sqrt(-2 ln u) cos(2 pi v), z_b = sqrt(-2 ln u) sin(2 pi v) with   */
/*   u = ((w_a >> 8) + 1) / 2^24 in (0, 1], v = (w_b >> 8) / 2^24 in [0, 1); */
/*   ln by range reduction to [sqrt(1/2), sqrt(2)] and the atanh series,     */
/*   cos / sin by octant and the Taylor polynomials on [0, pi/4).            */

static float f32_from_bits(uint32_t b) { float f; memcpy(&f, &b, 4); return f; }
static uint32_t f32_bits(float f) { uint32_t b; memcpy(&b, &f, 4); return b; }

/* -ln(n / 2^24) for an integer n in [1, 2^24], in binary32 steps. */
float isr_oracle_neg_log_u24(uint32_t n) {
    float f = (float)n;                       /* exact: n <= 2^24 */
    uint32_t bits = f32_bits(f);
    int32_t E = (int32_t)(bits >> 23) - 127;  /* n = m 2^E, m in [1, 2) */
    float m = f32_from_bits((bits & 0x7FFFFFu) | 0x3F800000u);
    if (m > 1.41421354f) { m = m * 0.5f; E += 1; }
    float k = (float)(24 - E);
    float s = (m - 1.0f) / (m + 1.0f);        /* ln m = 2 atanh(s), |s| <= 0.1716 */
    float s2 = s * s;
    float p = 0.222222224f;                   /* 2/9 */
    p = p * s2; p = p + 0.285714298f;         /* 2/7 */
    p = p * s2; p = p + 0.400000006f;         /* 2/5 */
    p = p * s2; p = p + 0.666666687f;         /* 2/3 */
    p = p * s2; p = p + 2.0f;
    float lnm = s * p;
    float a = k * 0.693145752f;               /* ln 2 = hi + lo; k * hi is exact */
    float b = k * 1.42860677e-06f;
    float d = a - lnm;
    return d + b;
}

/* cos and sin of the angle 2 pi t / 2^24, t in [0, 2^24), in binary32 steps. */
void isr_oracle_cos_sin_turn24(uint32_t t, float *cos_out, float *sin_out) {
    uint32_t octant = t >> 21, q = t & 0x1FFFFFu;
    float phi = (float)q * 3.74507039e-07f;   /* (pi/4) / 2^21: phi in [0, pi/4) */
    float x2 = phi * phi;
    float c = -2.755732e-07f;                 /* -1/10! */
    c = c * x2; c = c + 2.48015876e-05f;      /*  1/8!  */
    c = c * x2; c = c - 0.00138888892f;       /* -1/6!  */
    c = c * x2; c = c + 0.0416666679f;        /*  1/4!  */
    c = c * x2; c = c - 0.5f;
    c = c * x2; c = c + 1.0f;
    float s = 2.75573188e-06f;                /*  1/9!  */
    s = s * x2; s = s - 0.000198412701f;      /* -1/7!  */
    s = s * x2; s = s + 0.00833333377f;       /*  1/5!  */
    s = s * x2; s = s - 0.166666672f;         /* -1/3!  */
    s = s * x2; s = s + 1.0f;
    s = s * phi;
    float d = c - s, e = c + s;
    d = d * 0.707106769f;                     /* cos(pi/4 + phi) */
    e = e * 0.707106769f;                     /* sin(pi/4 + phi) */
    switch (octant) {
    case 0: *cos_out = c; *sin_out = s; break;
    case 1: *cos_out = d; *sin_out = e; break;
    case 2: *cos_out = -s; *sin_out = c; break;
    case 3: *cos_out = -e; *sin_out = d; break;
    case 4: *cos_out = -c; *sin_out = -s; break;
    case 5: *cos_out = -d; *sin_out = -e; break;
    case 6: *cos_out = s; *sin_out = -c; break;
    default: *cos_out = e; *sin_out = -d; break;
    }
}

/* The Box-Muller pair of two 32-bit words. */
void isr_oracle_box_muller(uint32_t wa, uint32_t wb, float *za, float *zb) {
    float l = isr_oracle_neg_log_u24((wa >> 8) + 1u);
    float r = sqrtf(2.0f * l);
    float c, s;
    isr_oracle_cos_sin_turn24(wb >> 8, &c, &s);
    *za = r * c;
    *zb = r * s;
}

/* The four standard-normal draws of elements 4 group .. 4 group + 3 of one noisy copy. */
void isr_oracle_gauss4(uint64_t seed, uint32_t image, uint32_t phase, uint32_t sample, uint32_t group, float z[4]) {
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t ctr[4] = {group, sample, image, 8u + phase};
    uint32_t w[4];
    isr_oracle_philox4x32_10(ctr, key, w);
    isr_oracle_box_muller(w[0], w[1], &z[0], &z[1]);
    isr_oracle_box_muller(w[2], w[3], &z[2], &z[3]);
}

/* v = x + sigma z for every element of one noisy copy (binary32: one product, one sum). */
void isr_oracle_noisy_float(const uint8_t *x, uint32_t npix, float sigma, uint64_t seed, uint32_t image,
                            uint32_t phase, uint32_t sample, float *v) {
    for (uint32_t p = 0; p < npix; ++p) {
        float z[4];
        isr_oracle_gauss4(seed, image, phase, sample, p >> 2, z);
        float sz = sigma * z[p & 3];
        v[p] = (float)x[p] + sz;
    }
}

/* FloatRS-quant input: the noisy value rounded to the nearest pixel level (ties to even),
 * saturated to [0, 255], recentred like the integer path's input. */
void isr_oracle_noisy_quant(const uint8_t *x, uint32_t npix, float sigma, uint64_t seed, uint32_t image,
                            uint32_t phase, uint32_t sample, int8_t *a0) {
    float *v = (float *)malloc((size_t)npix * sizeof(float));
    isr_oracle_noisy_float(x, npix, sigma, seed, image, phase, sample, v);
    for (uint32_t p = 0; p < npix; ++p) {
        float r = rintf(v[p]);
        if (r < 0.0f) r = 0.0f;
        if (r > 255.0f) r = 255.0f;
        a0[p] = (int8_t)((int32_t)r - 128);
    }
    free(v);
}

/* The float network behind a quantized one: every tensor holds the real values r = q - z that
 * the int8 codes stand for, every op is the quantized op without its rounding and without its
 * saturation at the ends of the int8 range (a ReLU stays: the lower clamp at the zero-point is
 * r >= 0):
 *   CONV     r_out = act(M (bias + sum over in-bounds taps of r_in w)), M = M0 2^-(31 + shift)
 *   ADD      r_out = act((Ma r_a + Mb r_b) 2^-shift)
 *   MAXPOOL  max over in-bounds taps;   GAP  r_out = M sum over H x W of r_in
 *   FC       logits = bias + sum r_in w
 * evaluated here in binary64.  The input is r_0 = v - 128 - z_0 for the noisy pixel values v. */
static double act(double v, int32_t relu) { return relu && v < 0.0 ? 0.0 : v; }

int isr_oracle_forward_float(const omodel *m, const float *v, double *acts, double *logits) {
    size_t *off = (size_t *)malloc((size_t)m->nt * sizeof(size_t));
    for (int i = 0; i < m->nt; ++i) off[i] = isr_oracle_tensor_offset(m, i);
    size_t n0 = (size_t)m->C * m->H * m->W;
    for (size_t i = 0; i < n0; ++i) acts[i] = (double)v[i] - 128.0 - (double)m->t[0].zp;
    for (int i = 0; i < m->nops; ++i) {
        const oop *o = &m->ops[i];
        otensor ti = m->t[o->a], to = m->t[o->out];
        const double *in = acts + off[o->a];
        double *out = acts + off[o->out];
        switch (o->type) {
        case OP_CONV:
            for (int oc = 0; oc < to.C; ++oc) {
                double M = ldexp((double)o->M0[oc], -(31 + o->shift[oc]));
                for (int oy = 0; oy < to.H; ++oy)
                    for (int ox = 0; ox < to.W; ++ox) {
                        double acc = (double)o->bias[oc];
                        for (int ic = 0; ic < ti.C; ++ic)
                            for (int ky = 0; ky < o->k; ++ky) {
                                int iy = oy * o->stride - o->pad + ky;
                                if (iy < 0 || iy >= ti.H) continue;
                                for (int kx = 0; kx < o->k; ++kx) {
                                    int ix = ox * o->stride - o->pad + kx;
                                    if (ix < 0 || ix >= ti.W) continue;
                                    acc += in[((size_t)ic * ti.H + iy) * ti.W + ix] *
                                           (double)o->w[(((size_t)oc * ti.C + ic) * o->k + ky) * o->k + kx];
                                }
                            }
                        out[((size_t)oc * to.H + oy) * to.W + ox] = act(acc * M, o->relu);
                    }
            }
            break;
        case OP_ADD: {
            const double *b = acts + off[o->b];
            size_t n = (size_t)to.C * to.H * to.W;
            for (size_t j = 0; j < n; ++j)
                out[j] = act(ldexp(in[j] * (double)o->Ma + b[j] * (double)o->Mb, -o->sh), o->relu);
            break; }
        case OP_MAXPOOL:
            for (int c = 0; c < to.C; ++c)
                for (int oy = 0; oy < to.H; ++oy)
                    for (int ox = 0; ox < to.W; ++ox) {
                        double best = 0.0;
                        int any = 0;
                        for (int ky = 0; ky < o->k; ++ky)
                            for (int kx = 0; kx < o->k; ++kx) {
                                int iy = oy * o->stride - o->pad + ky, ix = ox * o->stride - o->pad + kx;
                                if (iy < 0 || iy >= ti.H || ix < 0 || ix >= ti.W) continue;
                                double q = in[((size_t)c * ti.H + iy) * ti.W + ix];
                                if (!any || q > best) { best = q; any = 1; }
                            }
                        out[((size_t)c * to.H + oy) * to.W + ox] = best;
                    }
            break;
        case OP_GAP:
            for (int c = 0; c < ti.C; ++c) {
                double S = 0.0;
                for (int j = 0; j < ti.H * ti.W; ++j) S += in[(size_t)c * ti.H * ti.W + j];
                out[c] = S * ldexp((double)o->Ma, -(31 + o->sh));
            }
            break;
        case OP_FC: {
            int cin = ti.C * ti.H * ti.W;
            for (int oc = 0; oc < to.C; ++oc) {
                double acc = (double)o->bias[oc];
                for (int j = 0; j < cin; ++j) acc += in[j] * (double)o->w[(size_t)oc * cin + j];
                logits[oc] = acc;
            }
            break; }
        }
    }
    free(off);
    return 0;
}

/* Monte-Carlo loop of a comparison system over sample indices [begin, begin + count) of one
 * phase.  variant 1 = FloatRS-quant (int32 logits into logits_i), 2 = FloatRS-fp (binary64
 * logits into logits_d); the unused logits pointer, argmax and counts may be NULL. */
int isr_oracle_mc_float(const omodel *m, const uint8_t *x, float sigma, uint64_t seed, uint32_t image,
                        uint32_t phase, uint32_t begin, uint32_t count, int variant, int32_t *logits_i,
                        double *logits_d, int32_t *argmax, uint32_t *counts, int threads) {
    if (variant != 1 && variant != 2) return -1;
    uint32_t npix = (uint32_t)(m->C * m->H * m->W);
    size_t total = isr_oracle_tensor_offset(m, m->nt);
    int32_t *am = (int32_t *)malloc((size_t)count * sizeof(int32_t));
    if (threads < 1) threads = 1;
#pragma omp parallel num_threads(threads)
    {
        int8_t *a0 = (int8_t *)malloc(npix);
        float *v = (float *)malloc((size_t)npix * sizeof(float));
        int8_t *acts = (int8_t *)malloc(variant == 1 ? total : 1);
        double *facts = (double *)malloc((variant == 2 ? total : 1) * sizeof(double));
        int32_t *lg = (int32_t *)malloc((size_t)m->classes * sizeof(int32_t));
        double *lf = (double *)malloc((size_t)m->classes * sizeof(double));
#pragma omp for schedule(dynamic, 1)
        for (uint32_t s = 0; s < count; ++s) {
            if (variant == 1) {
                isr_oracle_noisy_quant(x, npix, sigma, seed, image, phase, begin + s, a0);
                isr_oracle_forward(m, a0, acts, lg);
                am[s] = isr_oracle_argmax(lg, m->classes);
                if (logits_i) memcpy(logits_i + (size_t)s * m->classes, lg, (size_t)m->classes * sizeof(int32_t));
            } else {
                isr_oracle_noisy_float(x, npix, sigma, seed, image, phase, begin + s, v);
                isr_oracle_forward_float(m, v, facts, lf);
                int32_t best = 0;
                for (int32_t c = 1; c < m->classes; ++c) if (lf[c] > lf[best]) best = c;
                am[s] = best;
                if (logits_d) memcpy(logits_d + (size_t)s * m->classes, lf, (size_t)m->classes * sizeof(double));
            }
        }
        free(a0); free(v); free(acts); free(facts); free(lg); free(lf);
    }
    for (uint32_t s = 0; s < count; ++s) {
        if (argmax) argmax[s] = am[s];
        if (counts) counts[am[s]] += 1;
    }
    free(am);
    return 0;
}
