/* Drives the CPU oracle (oracle/sco.c, included below) through every storage type, trigger
 * policy, threshold mode and record mode with seeded inputs.  Built by
 * tests/test_oracle_sanitizers.py with -fsanitize=address,undefined: any out-of-bounds access,
 * use after free, leak, signed overflow or misaligned access in the oracle ends the run with a
 * non-zero status.  Prints a checksum so that the run cannot be optimised away. */
#include "../../oracle/sco.c"

#include <stdio.h>

static uint32_t rng_state = 12345u;
static float rnd(void) { /* uniform in [-1, 1) */
    rng_state = rng_state * 1664525u + 1013904223u;
    return (float)(rng_state >> 8) / 8388608.0f - 1.0f;
}

static uint16_t to_half_bits(float f) {
    /* values in [-1, 1) with few mantissa bits convert exactly: keep 8 bits */
    const float q = (float)((int)(f * 128.0f)) / 128.0f;
    uint32_t u;
    memcpy(&u, &q, 4);
    const uint32_t sign = (u >> 16) & 0x8000u;
    const int32_t e = (int32_t)((u >> 23) & 0xffu) - 127 + 15;
    if (q == 0.0f || e <= 0) return (uint16_t)sign;
    return (uint16_t)(sign | ((uint32_t)e << 10) | ((u >> 13) & 0x3ffu));
}

static double run_case(int kv, int d, int trigger, int thresh, int record, int B, int r, int w, int m,
                       int steps) {
    sco_config cfg;
    memset(&cfg, 0, sizeof(cfg));
    cfg.batch = 2;
    cfg.heads = 2;
    cfg.head_dim = d;
    cfg.kv_dtype = kv;
    cfg.budget = B;
    cfg.recent = r;
    cfg.history = w;
    cfg.drop = m;
    cfg.trigger = trigger;
    cfg.thresh_mode = thresh;
    cfg.scale = 0.0;
    cfg.record_mode = record;
    sco_cache *h = sco_create(&cfg, 3);
    if (!h) {
        fprintf(stderr, "configuration rejected\n");
        exit(3);
    }
    int32_t n, cap;
    int64_t t;
    sco_len(h, &n, &t, &cap);
    const int U = 4;
    const size_t esz = kv == SCO_F32 ? 4 : 2;
    void *q = malloc((size_t)U * d * esz), *k = malloc((size_t)U * d * esz), *v = malloc((size_t)U * d * esz);
    double *out = malloc(sizeof(double) * (size_t)U * d);
    double *probs = malloc(sizeof(double) * (size_t)U * cap);
    int32_t *ev = malloc(sizeof(int32_t) * (size_t)U * m);
    int32_t *I = malloc(sizeof(int32_t) * (size_t)U * cap);
    int64_t *pos = malloc(sizeof(int64_t) * (size_t)U * cap);
    float *Kr = malloc(sizeof(float) * (size_t)U * cap * d), *Vr = malloc(sizeof(float) * (size_t)U * cap * d);
    double sum = 0.0;
    for (int s = 0; s < steps; ++s) {
        for (int i = 0; i < U * d; ++i) {
            const float a = rnd(), b = rnd(), c = rnd();
            if (kv == SCO_F32) {
                ((float *)q)[i] = a;
                ((float *)k)[i] = b;
                ((float *)v)[i] = c;
            } else {
                ((uint16_t *)q)[i] = to_half_bits(a);
                ((uint16_t *)k)[i] = to_half_bits(b);
                ((uint16_t *)v)[i] = to_half_bits(c);
            }
        }
        int32_t due = 0;
        if (sco_step(h, q, k, v, out, (s & 1) ? probs : NULL, NULL, 0, &due)) exit(4);
        sum += out[0] + out[(size_t)U * d - 1];
        sco_importance(h, I);
        sco_positions(h, pos);
        if (due) {
            if (record == SCO_RECORD_RECOMPUTE) {
                if (sco_compress_recompute(h, ev, NULL, NULL, 0, I)) exit(5);
            } else if (sco_compress(h, (s & 2) ? ev : NULL)) {
                exit(5);
            }
            sco_rows(h, Kr, Vr);
            sco_len(h, &n, &t, &cap);
            sum += Kr[0] + Vr[(size_t)U * n * d - 1];
        }
    }
    sco_importance_online(h, I);
    sum += I[0];
    free(q); free(k); free(v); free(out); free(probs); free(ev); free(I); free(pos); free(Kr); free(Vr);
    sco_destroy(h);
    return sum;
}

int main(void) {
    double sum = 0.0;
    const int kvs[3] = {SCO_F32, SCO_F16, SCO_I4G64};
    for (int a = 0; a < 3; ++a)
        for (int trigger = 0; trigger < 2; ++trigger)
            for (int thresh = 0; thresh < 2; ++thresh)
                for (int record = 0; record < 2; ++record) {
                    const int d = (a + trigger) % 2 ? 128 : 64;
                    sum += run_case(kvs[a], d, trigger, thresh, record, 24, 3, 10, 5, 90);
                    sum += run_case(kvs[a], d, trigger, thresh, record, 7, 1, 33, 1, 40);
                    sum += run_case(kvs[a], d, trigger, thresh, record, 16, 16 - 7, 4, 8, 60);
                }
    uint8_t codes[128];
    uint16_t x[128], sc[2], zr[2];
    float stored[128];
    for (int i = 0; i < 128; ++i) x[i] = to_half_bits(rnd());
    if (sco_i4_roundtrip(x, 128, codes, sc, zr, stored)) return 6;
    sum += stored[5] + sco_half_to_float(x[3]);
    printf("checksum %.17g\n", sum);
    return 0;
}
