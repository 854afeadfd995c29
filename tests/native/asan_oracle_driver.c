/* Runs every function of the C oracle on small heap buffers of exactly the documented sizes, so
 * that a build with -fsanitize=address,undefined reports any access past an argument's end, any
 * misaligned or overflowing arithmetic and any leak.  Buffers are allocated with malloc (red
 * zones on both sides), one per argument.  Exit code 0 and nothing on stderr = clean. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void orc_set_num_threads(int n);
void orc_route(const uint16_t *x, const uint16_t *wr, const float *bias, int T, int H, int E, int k, int renormalize,
               int32_t *ids, double *w, double *conf, double *logits);
void orc_perm(const int32_t *ids, int n, int E, int32_t *count, int32_t *off, int32_t *perm);
void orc_union(const int32_t *ids, int n, int E, const int32_t *slot_of_expert, uint64_t *mask, int32_t *list,
               int32_t *n_list, int32_t *missing, int32_t *n_missing);
void orc_dequant(const uint8_t *q, const uint16_t *s, const uint16_t *z, int R, int C, int g, double *out);
void orc_ffn_bf16(const uint16_t *wg, const uint16_t *wu, const uint16_t *wd, int H, int I, const double *x, double *out);
void orc_ffn_int4(const uint8_t *qg, const uint16_t *sg, const uint16_t *zg, const uint8_t *qu, const uint16_t *su,
                  const uint16_t *zu, const uint8_t *qd, const uint16_t *sd, const uint16_t *zd, int H, int I, int g,
                  const double *x, double *out);
void orc_layer_bf16(const uint16_t *x, const uint16_t *wg, const uint16_t *wu, const uint16_t *wd, int T, int H, int I,
                    int E, int S, int k, const int32_t *ids, const double *w, const uint8_t *present, double *y);
void orc_layer_int4(const uint16_t *x, const uint8_t *qg, const uint16_t *sg, const uint16_t *zg, const uint8_t *qu,
                    const uint16_t *su, const uint16_t *zu, const uint8_t *qd, const uint16_t *sd, const uint16_t *zd,
                    const uint16_t *swg, const uint16_t *swu, const uint16_t *swd, int T, int H, int I, int E, int S,
                    int k, int g, const int32_t *ids, const double *w, double *y);

static uint32_t rng_state = 12345u;
static uint32_t rnd(void) { rng_state = rng_state * 1664525u + 1013904223u; return rng_state >> 8; }
/* small bf16 values: sign, exponent near 1, a few mantissa bits */
static uint16_t rnd_bf16(void) { return (uint16_t)(((rnd() & 1u) << 15) | ((120u + rnd() % 10u) << 7) | (rnd() & 0x7fu)); }
static uint16_t rnd_fp16_scale(void) { return (uint16_t)(((10u + rnd() % 6u) << 10) | (rnd() & 0x3ffu)); }   /* positive, small */
static uint16_t fp16_of_int(int v) { static const uint16_t t[16] = {0x0000, 0x3c00, 0x4000, 0x4200, 0x4400, 0x4500, 0x4600, 0x4700,
                                                                    0x4800, 0x4880, 0x4900, 0x4980, 0x4a00, 0x4a80, 0x4b00, 0x4b80};
                                     return t[v & 15]; }

static uint16_t *bf16_buf(size_t n) { uint16_t *p = malloc(n * 2); for (size_t i = 0; i < n; ++i) p[i] = rnd_bf16(); return p; }
static uint8_t *code_buf(size_t n) { uint8_t *p = malloc(n); for (size_t i = 0; i < n; ++i) p[i] = (uint8_t)(rnd() & 15u); return p; }
static uint16_t *scale_buf(size_t n) { uint16_t *p = malloc(n * 2); for (size_t i = 0; i < n; ++i) p[i] = rnd_fp16_scale(); return p; }
static uint16_t *zero_buf(size_t n) { uint16_t *p = malloc(n * 2); for (size_t i = 0; i < n; ++i) p[i] = fp16_of_int((int)(rnd() & 15u)); return p; }

static int run_case(int T, int H, int E, int I, int k, int g, int S, int renorm, int with_bias)
{
    const size_t n = (size_t)T * k;
    uint16_t *x = bf16_buf((size_t)T * H), *wr = bf16_buf((size_t)E * H);
    float *bias = with_bias ? malloc(sizeof(float) * E) : NULL;
    for (int e = 0; bias && e < E; ++e) bias[e] = (float)(rnd() % 7) * 0.25f;
    int32_t *ids = malloc(sizeof(int32_t) * n);
    double *w = malloc(sizeof(double) * n), *conf = malloc(sizeof(double) * n), *logits = malloc(sizeof(double) * (size_t)T * E);
    orc_route(x, wr, bias, T, H, E, k, renorm, ids, w, conf, logits);
    for (size_t a = 0; a < n; ++a) if (ids[a] < 0 || ids[a] >= E) { fprintf(stderr, "bad id\n"); return 1; }

    int32_t *count = malloc(sizeof(int32_t) * E), *off = malloc(sizeof(int32_t) * (E + 1)), *perm = malloc(sizeof(int32_t) * n);
    orc_perm(ids, (int)n, E, count, off, perm);
    if (off[E] != (int32_t)n) { fprintf(stderr, "bad offsets\n"); return 1; }

    int32_t *slot = malloc(sizeof(int32_t) * E);
    for (int e = 0; e < E; ++e) slot[e] = (e % 3 == 0) ? -1 : e;
    uint64_t *mask = malloc(sizeof(uint64_t) * ((E + 63) / 64));
    int32_t *list = malloc(sizeof(int32_t) * E), *missing = malloc(sizeof(int32_t) * E), n_list = -1, n_missing = -1;
    orc_union(ids, (int)n, E, slot, mask, list, &n_list, missing, &n_missing);
    orc_union(ids, (int)n, E, NULL, mask, list, &n_list, NULL, &n_missing);
    orc_union(ids, 0, E, slot, mask, list, &n_list, missing, &n_missing);           /* empty window */

    const size_t P = (size_t)H * I, ES = (size_t)(E + S);
    uint16_t *wg = bf16_buf(ES * P), *wu = bf16_buf(ES * P), *wd = bf16_buf(ES * P);
    uint8_t *present = malloc(E);
    for (int e = 0; e < E; ++e) present[e] = (uint8_t)(e % 2);
    double *y = malloc(sizeof(double) * (size_t)T * H);
    orc_layer_bf16(x, wg, wu, wd, T, H, I, E, S, k, ids, w, NULL, y);
    orc_layer_bf16(x, wg, wu, wd, T, H, I, E, S, k, ids, w, present, y);

    uint8_t *qg = code_buf((size_t)E * P), *qu = code_buf((size_t)E * P), *qd = code_buf((size_t)E * P);
    uint16_t *sg = scale_buf((size_t)E * I * (H / g)), *su = scale_buf((size_t)E * I * (H / g)), *sd = scale_buf((size_t)E * H * (I / g));
    uint16_t *zg = zero_buf((size_t)E * I * (H / g)), *zu = zero_buf((size_t)E * I * (H / g)), *zd = zero_buf((size_t)E * H * (I / g));
    orc_layer_int4(x, qg, sg, zg, qu, su, zu, qd, sd, zd, S ? wg + (size_t)E * P : NULL, S ? wu + (size_t)E * P : NULL,
                   S ? wd + (size_t)E * P : NULL, T, H, I, E, S, k, g, ids, w, y);

    double *xv = malloc(sizeof(double) * H), *o = malloc(sizeof(double) * H), *deq = malloc(sizeof(double) * P);
    for (int h = 0; h < H; ++h) xv[h] = (double)(rnd() % 17) - 8.0;
    orc_ffn_bf16(wg, wu, wd, H, I, xv, o);
    orc_ffn_int4(qg, sg, zg, qu, su, zu, qd, sd, zd, H, I, g, xv, o);
    orc_dequant(qg, sg, zg, I, H, g, deq);
    orc_dequant(qd, sd, zd, H, I, g, deq);
    for (int h = 0; h < H; ++h) if (!(o[h] == o[h])) { fprintf(stderr, "nan\n"); return 1; }

    free(x); free(wr); free(bias); free(ids); free(w); free(conf); free(logits); free(count); free(off); free(perm);
    free(slot); free(mask); free(list); free(missing); free(wg); free(wu); free(wd); free(present); free(y);
    free(qg); free(qu); free(qd); free(sg); free(su); free(sd); free(zg); free(zu); free(zd); free(xv); free(o); free(deq);
    return 0;
}

int main(void)
{
    int rc = 0;
    for (int threads = 1; threads <= 3; threads += 2) {
        orc_set_num_threads(threads);
        rc |= run_case(1, 64, 4, 64, 1, 32, 0, 1, 0);         /* smallest shapes */
        rc |= run_case(3, 128, 5, 64, 2, 64, 1, 1, 1);        /* E not a power of two, one shared expert, bias */
        rc |= run_case(5, 192, 70, 128, 3, 32, 0, 0, 0);      /* more than 64 experts (two mask words), no renormalisation */
        rc |= run_case(2, 128, 130, 128, 16, 128, 2, 1, 1);   /* three mask words, k = 16, g = H */
        rc |= run_case(4, 64, 8, 64, 8, 32, 0, 1, 0);         /* k = E */
    }
    if (rc == 0) printf("oracle driver: ok\n");
    return rc;
}
