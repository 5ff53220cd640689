/*
 * sco.c — CPU oracle for the budgeted KV cache of Scissorhands (arxiv 2305.17118).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the GPU
 * library is checked against.  It shares no code, header, table or helper with the
 * HIP path and must never be linked into, imported by or called from the product.
 * Only the tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What it computes, per independent (sequence, head) unit, all arithmetic in double:
 *
 *   step      Alg. 1 loop body ("model update" appends one K/V row, n <- n+1), then the
 *             budgeted attention estimator of Sec. 4.1 over the n resident rows
 *             (scores, softmax, weighted sum of value rows), then one update of the
 *             importance record of Alg. 2 kept online as Sec. 4.1 "Overhead Tradeoff"
 *             allows: a row is "low" at this step when its probability is below the
 *             threshold 1/t; the low flags of the last w steps are kept per row.
 *             (Alg. 2 as printed instead recomputes the record at compression time with
 *             "an extra attention computation": record mode "recompute", below.)
 *   compress  Alg. 2: importance I = number of low flags inside the history window,
 *             the r most recent rows are not candidates, the m candidates with the
 *             largest I are dropped (equal I: the lowest slot goes first), survivors
 *             keep their order, n <- n-m.
 *
 * Readings taken where the paper is silent or inconsistent:
 *   - score = scale * <q, k_j>, q/k/v handed in by the caller, scale defaults to
 *     1/sqrt(head_dim); the sum runs over every resident row including the row
 *     appended at this step (Sec. 4.1 sums i = 1..t).
 *   - the history window is the last w steps, (t-w, t]; rows younger than w simply
 *     have fewer observations.
 *   - threshold 1/t with t = tokens seen including the current one, evaluated in
 *     fp32 (tau = 1.0f/(float)t) on the fp32 value of the probability, strict "<".
 *     Optional mode: 1/n (resident rows).
 *   - trigger: "hard cap" compresses when n == B+1 (Alg. 1 "if n > B"), leaving
 *     B+1-m rows; "high water" compresses when n == B+m, leaving exactly B rows.
 *   - record mode "recompute" (Alg. 2 literal; Sec. 4.1 "Overhead Tradeoff" names the extra
 *     attention computation): the queries of the last w steps are kept; at a compression
 *     at step t, for every step i in (t-w, t] the attention of q_i is recomputed over the
 *     rows resident NOW that step i could see (original position <= i-1), softmax over
 *     exactly those rows, and a row is low for step i when that probability is below
 *     1/i (or 1/(number of those rows) in the 1/n mode); I = number of low flags.  It
 *     differs from the online record only in that evicted rows no longer take part in
 *     the old queries' softmax.  A step none of whose rows survive contributes nothing.
 *   - 4-bit storage (Table 3 only names it): per row and per group of 64 channels,
 *     asymmetric: zero = min, scale = fp16(max-min)/15 (1 if that is 0),
 *     code = clamp(rint((x-zero)/scale), 0, 15) in fp32; the stored value is
 *     (float)code*scale + zero.  A row is quantised once, at append.
 *
 * Parity pins (tests/test_oracle_*.py): B >= T reduces to textbook softmax attention
 * (numpy and torch CPU), probabilities sum to 1, size and recent-window invariants,
 * brute-force subset enumeration for the selection, the restricted-softmax identity
 * used in the proof of Lemma A.4, closed-form counter cases, int4 round-trip bound.
 * Unpinned by the paper (fixed by this repository's readings): tie order, the exact
 * threshold variant, trigger policy, streaming prefill.
 */
#include <math.h>
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { SCO_F32 = 0, SCO_F16 = 1, SCO_I4G64 = 2 };
enum { SCO_HARD_CAP = 0, SCO_HIGH_WATER = 1 };
enum { SCO_INV_POS = 0, SCO_INV_LEN = 1 };
enum { SCO_RECORD_ONLINE = 0, SCO_RECORD_RECOMPUTE = 1 };

typedef struct {
    int32_t batch, heads, head_dim;
    int32_t kv_dtype;
    int32_t budget, recent, history, drop;
    int32_t trigger, thresh_mode;
    double scale; /* 0 -> 1/sqrt(head_dim) */
    int32_t record_mode;
} sco_config;

typedef struct sco_cache {
    sco_config cfg;
    int U, d, cap, w, r, m;
    int n;      /* resident rows, same for every unit */
    int64_t t;  /* tokens seen so far */
    double scale;
    float *K, *V;   /* [U][cap][d] stored values; every storage format is exact in fp32 */
    int64_t *pos;   /* [U][cap] original position (0-based) of the row in each slot */
    uint8_t *low;   /* [U][cap][w] ring: low[.][.][s % w] = flag written at step s */
    float *Qh;      /* [U][w][d] ring: Qh[.][s % w] = query of step s (as handed in) */
    int nthreads;
} sco_cache;

/* ---------- fp16 bit conversions (IEEE binary16, round to nearest even) ---------- */

static float half_bits_to_float(uint16_t h) {
    uint32_t sign = (uint32_t)(h >> 15) & 1u;
    int32_t ex = (h >> 10) & 0x1f;
    uint32_t man = h & 0x3ffu;
    double v;
    if (ex == 0) v = ldexp((double)man, -24);
    else if (ex == 31) v = man ? NAN : INFINITY;
    else v = ldexp((double)(man | 0x400u), ex - 25);
    return (float)(sign ? -v : v);
}

static uint16_t float_to_half_bits(float f) {
    uint32_t x;
    memcpy(&x, &f, 4);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    uint32_t ax = x & 0x7fffffffu;
    if (ax >= 0x7f800000u) return (uint16_t)(sign | (ax > 0x7f800000u ? 0x7e00u : 0x7c00u));
    double a = fabs((double)f);
    if (a == 0.0) return sign;
    int e;
    (void)frexp(a, &e); /* a = frac * 2^e, frac in [0.5,1) -> exponent of leading bit is e-1 */
    int lead = e - 1;
    if (lead < -14) lead = -14; /* subnormal range shares the spacing 2^-24 */
    double ulp = ldexp(1.0, lead - 10);
    double q = nearbyint(a / ulp); /* default rounding mode: nearest, ties to even */
    double r = q * ulp;
    if (r >= 65520.0) return (uint16_t)(sign | 0x7c00u);
    if (r < ldexp(1.0, -14)) return (uint16_t)(sign | (uint16_t)q); /* subnormal or zero */
    int e2;
    double fr = frexp(r, &e2); /* r = fr*2^e2 */
    uint32_t mant = (uint32_t)nearbyint(ldexp(fr, 11)) - 1024u;
    uint32_t bex = (uint32_t)(e2 - 1 + 15);
    return (uint16_t)(sign | (bex << 10) | mant);
}

/* ---------- 4-bit asymmetric group quantisation (group = 64 channels) ---------- */

/* Quantise one group of 64 fp32 values (which hold fp16 inputs exactly).  All
 * operations are single fp32 IEEE operations, so any conforming implementation
 * reproduces the codes bit for bit. */
static void i4_quant_group(const float *x, uint8_t *code, uint16_t *scale_h, uint16_t *zero_h) {
    float mn = x[0], mx = x[0];
    for (int c = 1; c < 64; ++c) {
        if (x[c] < mn) mn = x[c];
        if (x[c] > mx) mx = x[c];
    }
    volatile float range = mx - mn;
    volatile float sc = range / 15.0f;
    uint16_t sh = float_to_half_bits(sc);
    float s = half_bits_to_float(sh);
    if (s == 0.0f) {
        s = 1.0f;
        sh = 0x3c00u;
    }
    uint16_t zh = float_to_half_bits(mn); /* exact: mn is an fp16 value */
    float z = half_bits_to_float(zh);
    for (int c = 0; c < 64; ++c) {
        volatile float dlt = x[c] - z;
        volatile float qv = dlt / s;
        float rq = nearbyintf(qv);
        if (rq < 0.0f) rq = 0.0f;
        if (rq > 15.0f) rq = 15.0f;
        code[c] = (uint8_t)rq;
    }
    *scale_h = sh;
    *zero_h = zh;
}

static float i4_dequant(uint8_t code, uint16_t scale_h, uint16_t zero_h) {
    volatile float prod = (float)code * half_bits_to_float(scale_h); /* exact: 4 x 11 bits */
    volatile float v = prod + half_bits_to_float(zero_h);
    return v;
}

/* Exposed for the storage-format tests: x_h [d] fp16 bits -> codes [d], scale/zero [d/64]
 * fp16 bits, stored [d] fp32 stored values. */
int sco_i4_roundtrip(const uint16_t *x_h, int d, uint8_t *codes, uint16_t *scale_h,
                     uint16_t *zero_h, float *stored) {
    if (d <= 0 || d % 64) return 1;
    float buf[64];
    for (int g = 0; g < d / 64; ++g) {
        for (int c = 0; c < 64; ++c) buf[c] = half_bits_to_float(x_h[g * 64 + c]);
        i4_quant_group(buf, codes + g * 64, scale_h + g, zero_h + g);
        for (int c = 0; c < 64; ++c)
            stored[g * 64 + c] = i4_dequant(codes[g * 64 + c], scale_h[g], zero_h[g]);
    }
    return 0;
}

/* Exposed so the tests can check the converters against numpy's float16. */
float sco_half_to_float(uint16_t h) { return half_bits_to_float(h); }
uint16_t sco_float_to_half(float f) { return float_to_half_bits(f); }

/* ---------- cache ---------- */

static int trigger_rows(const sco_config *c) {
    return c->trigger == SCO_HIGH_WATER ? c->budget + c->drop : c->budget + 1;
}

sco_cache *sco_create(const sco_config *cfg, int nthreads) {
    if (!cfg) return NULL;
    if (cfg->batch < 1 || cfg->heads < 1 || cfg->head_dim < 1) return NULL;
    if (cfg->kv_dtype < 0 || cfg->kv_dtype > 2) return NULL;
    if (cfg->kv_dtype == SCO_I4G64 && cfg->head_dim % 64) return NULL;
    if (cfg->budget < 1 || cfg->recent < 1 || cfg->history < 1 || cfg->drop < 1) return NULL;
    if (cfg->trigger < 0 || cfg->trigger > 1 || cfg->thresh_mode < 0 || cfg->thresh_mode > 1)
        return NULL;
    if (cfg->record_mode < 0 || cfg->record_mode > 1) return NULL;
    int cap = trigger_rows(cfg);
    if (cfg->drop > cap - cfg->recent) return NULL; /* not enough candidates to drop m */
    sco_cache *h = (sco_cache *)calloc(1, sizeof(*h));
    if (!h) return NULL;
    h->cfg = *cfg;
    h->U = cfg->batch * cfg->heads;
    h->d = cfg->head_dim;
    h->cap = cap;
    h->w = cfg->history;
    h->r = cfg->recent;
    h->m = cfg->drop;
    h->scale = cfg->scale != 0.0 ? cfg->scale : 1.0 / sqrt((double)cfg->head_dim);
    h->nthreads = nthreads < 1 ? 1 : nthreads;
    size_t rows = (size_t)h->U * (size_t)cap;
    h->K = (float *)calloc(rows * (size_t)h->d, sizeof(float));
    h->V = (float *)calloc(rows * (size_t)h->d, sizeof(float));
    h->pos = (int64_t *)calloc(rows, sizeof(int64_t));
    h->low = (uint8_t *)calloc(rows * (size_t)h->w, 1);
    h->Qh = (float *)calloc((size_t)h->U * (size_t)h->w * (size_t)h->d, sizeof(float));
    if (!h->K || !h->V || !h->pos || !h->low || !h->Qh) {
        free(h->K); free(h->V); free(h->pos); free(h->low); free(h->Qh); free(h);
        return NULL;
    }
    return h;
}

void sco_destroy(sco_cache *h) {
    if (!h) return;
    free(h->K); free(h->V); free(h->pos); free(h->low); free(h->Qh); free(h);
}

int sco_len(const sco_cache *h, int32_t *n, int64_t *t, int32_t *cap) {
    if (!h) return 1;
    if (n) *n = h->n;
    if (t) *t = h->t;
    if (cap) *cap = h->cap;
    return 0;
}

/* ---------- threading over units ---------- */

typedef struct {
    void (*fn)(void *ctx, int u);
    void *ctx;
    int u0, u1;
} span_job;

static void *span_main(void *arg) {
    span_job *j = (span_job *)arg;
    for (int u = j->u0; u < j->u1; ++u) j->fn(j->ctx, u);
    return NULL;
}

static void for_each_unit(const sco_cache *h, void (*fn)(void *, int), void *ctx) {
    int nt = h->nthreads < h->U ? h->nthreads : h->U;
    if (nt <= 1) {
        for (int u = 0; u < h->U; ++u) fn(ctx, u);
        return;
    }
    pthread_t *th = (pthread_t *)malloc(sizeof(pthread_t) * (size_t)nt);
    span_job *jobs = (span_job *)malloc(sizeof(span_job) * (size_t)nt);
    for (int i = 0; i < nt; ++i) {
        jobs[i].fn = fn;
        jobs[i].ctx = ctx;
        jobs[i].u0 = (int)((int64_t)h->U * i / nt);
        jobs[i].u1 = (int)((int64_t)h->U * (i + 1) / nt);
        pthread_create(&th[i], NULL, span_main, &jobs[i]);
    }
    for (int i = 0; i < nt; ++i) pthread_join(th[i], NULL);
    free(th);
    free(jobs);
}

/* ---------- step ---------- */

typedef struct {
    sco_cache *h;
    const void *q, *k_new, *v_new;
    double *out;            /* [U][d] */
    double *probs;          /* [U][cap] or NULL */
    const float *p_forced;  /* [U][ld_forced] or NULL */
    int ld_forced;
    int n_after;            /* resident rows including the appended one */
    int64_t t_after;
    float tau;
} step_ctx;

static float load_elem(const void *base, int kv_dtype, size_t idx) {
    if (kv_dtype == SCO_F32) return ((const float *)base)[idx];
    return half_bits_to_float(((const uint16_t *)base)[idx]);
}

static void store_row(const sco_cache *h, float *dst, const void *src, size_t off) {
    int d = h->d;
    if (h->cfg.kv_dtype != SCO_I4G64) {
        for (int c = 0; c < d; ++c) dst[c] = load_elem(src, h->cfg.kv_dtype, off + (size_t)c);
        return;
    }
    float buf[64];
    uint8_t code[64];
    uint16_t sh, zh;
    for (int g = 0; g < d / 64; ++g) {
        for (int c = 0; c < 64; ++c)
            buf[c] = half_bits_to_float(((const uint16_t *)src)[off + (size_t)(g * 64 + c)]);
        i4_quant_group(buf, code, &sh, &zh);
        for (int c = 0; c < 64; ++c) dst[g * 64 + c] = i4_dequant(code[c], sh, zh);
    }
}

/* Sec. 4.1 estimator, probability part: s[j] = softmax_j(scale * <q, k_j>) over the first n
 * rows of K (the query already widened to double). */
static void attention_probabilities(const sco_cache *h, const float *K, int n, const double *qd,
                                    double *s) {
    const int d = h->d;
    double mx = -INFINITY;
    for (int j = 0; j < n; ++j) {
        double acc = 0.0;
        for (int ch = 0; ch < d; ++ch) acc += qd[ch] * (double)K[(size_t)j * d + ch];
        s[j] = h->scale * acc;
        if (s[j] > mx) mx = s[j];
    }
    double denom = 0.0;
    for (int j = 0; j < n; ++j) {
        s[j] = exp(s[j] - mx);
        denom += s[j];
    }
    for (int j = 0; j < n; ++j) s[j] /= denom;
}

static void step_unit(void *vctx, int u) {
    step_ctx *c = (step_ctx *)vctx;
    sco_cache *h = c->h;
    const int d = h->d, cap = h->cap, w = h->w;
    const int n = c->n_after;
    const int slot = n - 1;
    float *K = h->K + (size_t)u * cap * d;
    float *V = h->V + (size_t)u * cap * d;
    int64_t *pos = h->pos + (size_t)u * cap;
    uint8_t *low = h->low + (size_t)u * cap * w;

    /* Alg. 1: the model appends this step's key/value row. */
    store_row(h, K + (size_t)slot * d, c->k_new, (size_t)u * d);
    store_row(h, V + (size_t)slot * d, c->v_new, (size_t)u * d);
    pos[slot] = c->t_after - 1;
    memset(low + (size_t)slot * w, 0, (size_t)w);

    /* Sec. 4.1 estimator: scores over resident rows, softmax, weighted value sum. */
    double *s = (double *)malloc(sizeof(double) * (size_t)(n + d));
    double *qd = s + n; /* this unit's query, widened once */
    for (int ch = 0; ch < d; ++ch)
        qd[ch] = (double)load_elem(c->q, h->cfg.kv_dtype == SCO_F32 ? SCO_F32 : SCO_F16,
                                   (size_t)u * d + (size_t)ch);
    float *qkeep = h->Qh + ((size_t)u * w + (size_t)(c->t_after % w)) * d;
    for (int ch = 0; ch < d; ++ch) qkeep[ch] = (float)qd[ch]; /* exact: the input is fp32 or fp16 */
    attention_probabilities(h, K, n, qd, s); /* s now holds the probabilities */
    double *o = c->out + (size_t)u * d;
    for (int ch = 0; ch < d; ++ch) o[ch] = 0.0;
    for (int j = 0; j < n; ++j)
        for (int ch = 0; ch < d; ++ch) o[ch] += s[j] * (double)V[(size_t)j * d + ch];
    if (c->probs) {
        double *pr = c->probs + (size_t)u * cap;
        for (int j = 0; j < n; ++j) pr[j] = s[j];
        for (int j = n; j < cap; ++j) pr[j] = 0.0;
    }

    /* Alg. 2 counter kept online: flag rows whose probability is below the threshold.
     * The decision is taken in fp32: on the forced probabilities when given, else on
     * this oracle's own probability rounded to fp32. */
    int ring = (int)(c->t_after % w);
    for (int j = 0; j < n; ++j) {
        float pj = c->p_forced ? c->p_forced[(size_t)u * c->ld_forced + j] : (float)s[j];
        low[(size_t)j * w + ring] = (uint8_t)(pj < c->tau);
    }
    free(s);
}

/* One decode step for every unit.
 * q, k_new, v_new: [U][d], fp32 for SCO_F32 storage, fp16 bit patterns otherwise.
 * out [U][d] double; probs [U][cap] double or NULL; p_forced [U][ld_forced] fp32 or NULL
 * (when given, the low-score flags are decided on these values instead of the oracle's).
 * due: set to 1 when the cache has reached its trigger size and must be compressed
 * before the next step.  Returns 0, or 1 on a bad call (null, or step while due). */
int sco_step(sco_cache *h, const void *q, const void *k_new, const void *v_new, double *out,
             double *probs, const float *p_forced, int ld_forced, int32_t *due) {
    if (!h || !q || !k_new || !v_new || !out) return 1;
    if (h->n >= h->cap) return 1;
    if (p_forced && ld_forced < h->n + 1) return 1;
    step_ctx c;
    c.h = h;
    c.q = q; c.k_new = k_new; c.v_new = v_new;
    c.out = out; c.probs = probs; c.p_forced = p_forced; c.ld_forced = ld_forced;
    c.n_after = h->n + 1;
    c.t_after = h->t + 1;
    c.tau = h->cfg.thresh_mode == SCO_INV_LEN ? 1.0f / (float)c.n_after : 1.0f / (float)c.t_after;
    for_each_unit(h, step_unit, &c);
    h->n = c.n_after;
    h->t = c.t_after;
    if (due) *due = (h->n == h->cap);
    return 0;
}

/* ---------- importance and compression ---------- */

static int importance_of(const sco_cache *h, int u, int j) {
    const uint8_t *f = h->low + ((size_t)u * h->cap + (size_t)j) * h->w;
    int acc = 0;
    for (int i = 0; i < h->w; ++i) acc += f[i];
    return acc;
}

/* Number of steps in the history window at the current step: min(w, t). */
static int window_steps(const sco_cache *h) { return h->t < (int64_t)h->w ? (int)h->t : h->w; }

/* Record mode "recompute" for one unit: I[0..n) from the kept queries and the rows resident
 * now.  Window entry k (0-based) is step i = t - W + 1 + k, W = window_steps.
 * probs (nullable) [W][cap] receives this oracle's probabilities (0 where a row is not
 * visible to the step); p_forced (nullable) [W][ld] replaces them in the low decision. */
static void recompute_record_unit(const sco_cache *h, int u, int *I, double *probs,
                                  const float *p_forced, int ld) {
    const int n = h->n, d = h->d, cap = h->cap, w = h->w;
    const int W = window_steps(h);
    const float *K = h->K + (size_t)u * cap * d;
    const int64_t *pos = h->pos + (size_t)u * cap;
    double *s = (double *)malloc(sizeof(double) * (size_t)(n + d));
    double *qd = s + n;
    for (int j = 0; j < n; ++j) I[j] = 0;
    for (int k = 0; k < W; ++k) {
        const int64_t i = h->t - W + 1 + k; /* the step whose query is replayed */
        const float *q = h->Qh + ((size_t)u * w + (size_t)(i % w)) * d;
        int vis = 0; /* rows are kept in order of position, so the visible ones come first */
        while (vis < n && pos[vis] <= i - 1) ++vis;
        if (probs)
            for (int j = 0; j < cap; ++j) probs[(size_t)k * cap + j] = 0.0;
        if (vis == 0) continue;
        for (int ch = 0; ch < d; ++ch) qd[ch] = (double)q[ch];
        attention_probabilities(h, K, vis, qd, s);
        const float tau = h->cfg.thresh_mode == SCO_INV_LEN ? 1.0f / (float)vis : 1.0f / (float)i;
        for (int j = 0; j < vis; ++j) {
            const double p = s[j];
            if (probs) probs[(size_t)k * cap + j] = p;
            const float pf = p_forced ? p_forced[(size_t)k * ld + j] : (float)p;
            I[j] += (pf < tau);
        }
    }
    free(s);
}

/* I [U][n]: importance record of every resident row over the current history window
 * (online flags, or recomputed from the kept queries, according to the record mode). */
int sco_importance(const sco_cache *h, int32_t *I) {
    if (!h || !I) return 1;
    for (int u = 0; u < h->U; ++u) {
        if (h->cfg.record_mode == SCO_RECORD_RECOMPUTE) {
            int *tmp = (int *)malloc(sizeof(int) * (size_t)h->n);
            recompute_record_unit(h, u, tmp, NULL, NULL, 0);
            for (int j = 0; j < h->n; ++j) I[(size_t)u * h->n + j] = tmp[j];
            free(tmp);
        } else {
            for (int j = 0; j < h->n; ++j) I[(size_t)u * h->n + j] = importance_of(h, u, j);
        }
    }
    return 0;
}

/* The online record whatever the mode (the flags are always kept): lets a test compare the
 * two records on the same run. */
int sco_importance_online(const sco_cache *h, int32_t *I) {
    if (!h || !I) return 1;
    for (int u = 0; u < h->U; ++u)
        for (int j = 0; j < h->n; ++j) I[(size_t)u * h->n + j] = importance_of(h, u, j);
    return 0;
}

/* pos [U][n]: original 0-based position of the row in each slot. */
int sco_positions(const sco_cache *h, int64_t *pos) {
    if (!h || !pos) return 1;
    for (int u = 0; u < h->U; ++u)
        memcpy(pos + (size_t)u * h->n, h->pos + (size_t)u * h->cap, sizeof(int64_t) * (size_t)h->n);
    return 0;
}

/* K, V [U][n][d]: stored (post storage rounding) values of the resident rows. */
int sco_rows(const sco_cache *h, float *K, float *V) {
    if (!h || !K || !V) return 1;
    size_t rowsz = (size_t)h->d;
    for (int u = 0; u < h->U; ++u) {
        memcpy(K + (size_t)u * h->n * rowsz, h->K + (size_t)u * h->cap * rowsz,
               sizeof(float) * (size_t)h->n * rowsz);
        memcpy(V + (size_t)u * h->n * rowsz, h->V + (size_t)u * h->cap * rowsz,
               sizeof(float) * (size_t)h->n * rowsz);
    }
    return 0;
}

typedef struct {
    sco_cache *h;
    int32_t *evicted; /* [U][m] or NULL */
    /* record mode "recompute" only (all nullable): */
    double *re_probs;        /* [U][W][cap] */
    const float *re_forced;  /* [U][W][re_ld] */
    int re_ld;
    int32_t *record_out;     /* [U][n] the record the selection used */
} compress_ctx;

static void compress_unit(void *vctx, int u) {
    compress_ctx *c = (compress_ctx *)vctx;
    sco_cache *h = c->h;
    const int n = h->n, d = h->d, cap = h->cap, w = h->w, m = h->m;
    const int ncand = n - h->r; /* the r most recent slots are never candidates */
    int *I = (int *)malloc(sizeof(int) * (size_t)n);
    uint8_t *gone = (uint8_t *)calloc((size_t)n, 1);
    if (h->cfg.record_mode == SCO_RECORD_RECOMPUTE) {
        const int W = window_steps(h);
        recompute_record_unit(h, u, I, c->re_probs ? c->re_probs + (size_t)u * W * cap : NULL,
                              c->re_forced ? c->re_forced + (size_t)u * W * c->re_ld : NULL, c->re_ld);
    } else {
        for (int j = 0; j < n; ++j) I[j] = importance_of(h, u, j);
    }
    if (c->record_out)
        for (int j = 0; j < n; ++j) c->record_out[(size_t)u * n + j] = I[j];
    /* Drop the m candidates with the largest record; equal records: lowest slot first. */
    for (int k = 0; k < m; ++k) {
        int best = -1;
        for (int j = 0; j < ncand; ++j) {
            if (gone[j]) continue;
            if (best < 0 || I[j] > I[best]) best = j;
        }
        gone[best] = 1;
    }
    float *K = h->K + (size_t)u * cap * d;
    float *V = h->V + (size_t)u * cap * d;
    int64_t *pos = h->pos + (size_t)u * cap;
    uint8_t *low = h->low + (size_t)u * cap * w;
    int dst = 0, ne = 0;
    for (int j = 0; j < n; ++j) {
        if (gone[j]) {
            if (c->evicted) c->evicted[(size_t)u * m + ne] = j;
            ++ne;
            continue;
        }
        if (dst != j) {
            memcpy(K + (size_t)dst * d, K + (size_t)j * d, sizeof(float) * (size_t)d);
            memcpy(V + (size_t)dst * d, V + (size_t)j * d, sizeof(float) * (size_t)d);
            pos[dst] = pos[j];
            memcpy(low + (size_t)dst * w, low + (size_t)j * w, (size_t)w);
        }
        ++dst;
    }
    free(I);
    free(gone);
}

static void run_compression(compress_ctx *c) {
    sco_cache *h = c->h;
    for_each_unit(h, compress_unit, c);
    h->n -= h->m;
}

/* Alg. 2.  Only legal when the last step reported due.  evicted [U][m] (nullable)
 * receives the dropped slots of each unit in ascending order (slot numbers before
 * compaction).  Returns 0, or 1 when not due. */
int sco_compress(sco_cache *h, int32_t *evicted) {
    if (!h) return 1;
    if (h->n != h->cap) return 1;
    compress_ctx c;
    memset(&c, 0, sizeof(c));
    c.h = h;
    c.evicted = evicted;
    run_compression(&c);
    return 0;
}

/* Alg. 2 in record mode "recompute", with the replayed attention exposed:
 * probs [U][W][cap] double (nullable) receives the oracle's probabilities of the W = min(w, t)
 * replayed steps (oldest first); p_forced [U][W][ld] fp32 (nullable) replaces them in the
 * low decision; record_out [U][n] (nullable) receives the record the selection used.
 * Returns 0, or 1 when not due or not in that mode. */
int sco_compress_recompute(sco_cache *h, int32_t *evicted, double *probs, const float *p_forced,
                           int ld, int32_t *record_out) {
    if (!h) return 1;
    if (h->n != h->cap || h->cfg.record_mode != SCO_RECORD_RECOMPUTE) return 1;
    if (p_forced && ld < h->n) return 1;
    compress_ctx c;
    memset(&c, 0, sizeof(c));
    c.h = h;
    c.evicted = evicted;
    c.re_probs = probs;
    c.re_forced = p_forced;
    c.re_ld = ld;
    c.record_out = record_out;
    run_compression(&c);
    return 0;
}
